// Consumer of the compacted cache: one decode step's attention over the retained entries of
// every head (Sec. 3.2, Eq. 3 restricted to the index set I_{l,h}).  The packed K and V rows of
// head hi sit at [offsets[hi], offsets[hi+1]); the G query heads of a group share them.
//   decode_partial - one workgroup per (head, block of 128 rows), one wave per 16 rows.  The work
//                    is a handful of dot products per row read (G queries), bound by the read of
//                    K and V, so there is no staging and no matrix core: a wave loads its 16 K
//                    rows and 16 V rows straight into registers, row-coalesced (a row is shared
//                    by `lanes per row` neighbouring lanes, 16 bytes each), forms the logits with
//                    a butterfly over those lanes, and - because K and V rows sit in the same
//                    lanes - weights its own V pieces without moving a probability.  The eight
//                    waves meet once, in LDS, to leave (max, sum, weighted values) per query head.
//   decode_combine - one workgroup per (query head, head): merges the blocks' partial results.
// Row counts live on the device (they are budgets), so the grid covers the longest possible
// head and workgroups beyond a head's rows exit at once.
#include "lukv_internal.hpp"

namespace lukv {

constexpr int kDecMaxGroup = 16;   // query heads per KV head the decode kernels take
constexpr int kDecRows = 128;      // rows per workgroup of decode_partial
constexpr int kDecWaves = 8;       // waves of that workgroup; each takes kDecRows / kDecWaves rows

struct DecGeom {
  int32_t n_layers, n_q_heads, n_kv_heads, group, n_seqs, max_blocks;
  float scale;
};

template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __uint_as_float((unsigned)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(x), CTRL, 0xf, 0xf, true));
}

// sum over the LPR (8, 16 or 32) neighbouring lanes that share a row, left in every one of them:
// swaps inside a quad, then the mirrored half row and row
template <int LPR>
__device__ __forceinline__ float row_allsum(float x) {
  x += dpp_f<0xB1>(x);                  // quad_perm [1,0,3,2]
  x += dpp_f<0x4E>(x);                  // quad_perm [2,3,0,1]
  x += dpp_f<0x141>(x);                 // row_half_mirror: lane i <-> 7 - i
  if (LPR >= 16) x += dpp_f<0x140>(x);  // row_mirror: lane i <-> 15 - i
  if (LPR >= 32) x += __shfl_xor(x, 16);
  return x;
}

// NG query heads at a time (blockIdx.z picks the NG-group when the GQA group is larger).
template <bool F32, int D, int NG>
__global__ __launch_bounds__(64 * kDecWaves) void decode_partial_kernel(DecGeom g, const char* q, const char* kp,
                                                             const char* vp, const int64_t* offsets,
                                                             float* part) {
  constexpr int R = kDecRows;
  constexpr int kEsize = F32 ? 4 : 2;
  constexpr int EPL = 16 / kEsize;               // elements in a lane's 16-byte piece
  constexpr int LPR = D / EPL;                   // lanes per row: 8, 16 or 32
  constexpr int RPL = 64 / LPR;                  // rows per load instruction of a wave
  constexpr int WR = kDecRows / kDecWaves;       // rows of a wave
  constexpr int NLD = WR / RPL;                  // loads that cover them
  constexpr int kRowBytes = D * kEsize;
  __shared__ float wm[kDecWaves][NG], wl[kDecWaves][NG];
  __shared__ float wacc[kDecWaves][NG][D];
  const int hi = blockIdx.y, blk = blockIdx.x, t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int64_t row_begin = offsets[hi] + (int64_t)blk * R;
  const int64_t rows_left = offsets[hi + 1] - row_begin;
  if (rows_left <= 0) return;
  const int n = rows_left < R ? (int)rows_left : R;
  const int G = g.group, g0 = blockIdx.z * NG;
  const int kvh = hi % g.n_kv_heads, layer = (hi / g.n_kv_heads) % g.n_layers;
  const int seq = hi / (g.n_kv_heads * g.n_layers);
  const int c = lane % LPR, j = lane / LPR;

  // Loads go out in the order their data is used - queries, K, V - so that the logits of the
  // first rows are formed while later rows are still on their way.
  // this lane's piece of every query (queries beyond the group are zero)
  u32x4 qraw[NG];
#pragma unroll
  for (int gq = 0; gq < NG; ++gq) {
    qraw[gq] = u32x4{0u, 0u, 0u, 0u};
    if (g0 + gq < G) {
      const int64_t row = (((int64_t)layer * g.n_q_heads + kvh * G + g0 + gq) * g.n_seqs + seq);
      qraw[gq] = *reinterpret_cast<const u32x4*>(q + row * kRowBytes + c * 16);
    }
  }
  // the wave's K and V rows (rows beyond the block are clamped to its last row and weighted 0)
  u32x4 kr[NLD], vr[NLD];
  auto row_off = [&](int u) {
    const int r = WR * wave + u * RPL + j;
    return (row_begin + (r < n ? r : n - 1)) * kRowBytes + c * 16;
  };
#pragma unroll
  for (int u = 0; u < NLD; ++u) kr[u] = *reinterpret_cast<const u32x4*>(kp + row_off(u));
#pragma unroll
  for (int u = 0; u < NLD; ++u) vr[u] = *reinterpret_cast<const u32x4*>(vp + row_off(u));
  // (every load above is issued before any arithmetic below: the scheduler may not sink them)
  __builtin_amdgcn_sched_barrier(0);
  auto piece = [](const u32x4& x, float* f) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      if constexpr (F32) f[e] = __uint_as_float(x[e]);
      else f[e] = __uint_as_float((e & 1) ? (x[e >> 1] & 0xFFFF0000u) : (x[e >> 1] << 16));
    }
  };
  float qf[NG][EPL];
#pragma unroll
  for (int gq = 0; gq < NG; ++gq) piece(qraw[gq], qf[gq]);

  // logits of the lane's rows (row u * RPL + j of the wave for load u), every lane of a row
  float sv[NG][NLD];
#pragma unroll
  for (int u = 0; u < NLD; ++u) {
    float kf[EPL];
    piece(kr[u], kf);
    const bool live = WR * wave + u * RPL + j < n;
#pragma unroll
    for (int gq = 0; gq < NG; ++gq) {
      float d = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) d = fmaf(qf[gq][e], kf[e], d);
      d = row_allsum<LPR>(d);
      sv[gq][u] = live ? d * g.scale : -INFINITY;
    }
  }
  // the wave's maximum per query, probabilities, and the p-weighted sum of the lane's V pieces
  float acc[NG][EPL], lsum[NG], mw[NG];
#pragma unroll
  for (int gq = 0; gq < NG; ++gq) {
    float m = sv[gq][0];
#pragma unroll
    for (int u = 1; u < NLD; ++u) m = fmaxf(m, sv[gq][u]);
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) m = fmaxf(m, __shfl_xor(m, o));
    mw[gq] = m;
    const float ms = m == -INFINITY ? 0.f : m;
    float l = 0.f;
#pragma unroll
    for (int u = 0; u < NLD; ++u) {
      sv[gq][u] = __expf(sv[gq][u] - ms);      // a row beyond the block: exp(-inf) = 0
      l += sv[gq][u];
    }
    lsum[gq] = l;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[gq][e] = 0.f;
  }
#pragma unroll
  for (int u = 0; u < NLD; ++u) {
    float vf[EPL];
    piece(vr[u], vf);
#pragma unroll
    for (int gq = 0; gq < NG; ++gq)
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[gq][e] = fmaf(sv[gq][u], vf[e], acc[gq][e]);
  }
  // lanes that hold the same piece of different rows: fixed-order sums over the row index j
#pragma unroll
  for (int gq = 0; gq < NG; ++gq) {
#pragma unroll
    for (int o = LPR; o < 64; o <<= 1) {
      lsum[gq] += __shfl_xor(lsum[gq], o);
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[gq][e] += __shfl_xor(acc[gq][e], o);
    }
  }
  if (j == 0) {
#pragma unroll
    for (int gq = 0; gq < NG; ++gq) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) wacc[wave][gq][c * EPL + e] = acc[gq][e];
      if (c == 0) {
        wm[wave][gq] = mw[gq];
        wl[wave][gq] = lsum[gq];
      }
    }
  }
  __syncthreads();
  // the waves' results under their common maximum (wave 0 always holds a live row)
  float* my_part = part + ((int64_t)hi * g.max_blocks + blk) * G * (D + 2);
  for (int o = t; o < NG * D; o += 64 * kDecWaves) {
    const int gq = o / D, x = o - gq * D;
    if (g0 + gq >= G) continue;
    float M = wm[0][gq];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) M = fmaxf(M, wm[w][gq]);
    float a = 0.f, l = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) {
      const float e = __expf(wm[w][gq] - M);    // exp(-inf) = 0 for a wave without rows
      a = fmaf(wacc[w][gq][x], e, a);
      l = fmaf(wl[w][gq], e, l);
    }
    float* dst = my_part + (g0 + gq) * (D + 2);
    dst[x] = a;
    if (x == 0) {
      dst[D] = M;
      dst[D + 1] = l;
    }
  }
}

// One workgroup per (query head of the group, head): the blocks' partial results are merged in
// one pass.  D threads own the columns and 1024 / D groups of them share the blocks; a group keeps
// a running maximum and rescales its sums when it grows (sixteen blocks' values in flight
// at a time), and the groups meet once in LDS.
template <int D, int R>
__global__ __launch_bounds__(1024) void decode_combine_kernel(DecGeom g, const int64_t* offsets, const float* part,
                                                              float* out) {
  constexpr int NP = 1024 / D;          // groups of D threads that share the blocks
  constexpr int U = 16;
  __shared__ float pm[NP], pl[NP];
  __shared__ float accs[NP][D];
  const int gq = blockIdx.x, hi = blockIdx.y, t = threadIdx.x;
  const int G = g.group;
  const int kvh = hi % g.n_kv_heads, layer = (hi / g.n_kv_heads) % g.n_layers;
  const int seq = hi / (g.n_kv_heads * g.n_layers);
  const int64_t rows = offsets[hi + 1] - offsets[hi];
  const int n_blk = (int)((rows + R - 1) / R);
  const float* hp = part + ((int64_t)hi * g.max_blocks * G + gq) * (D + 2);
  const int64_t bstride = (int64_t)G * (D + 2);
  const int x = t % D, pt = t / D;
  float* dst = out + (((int64_t)layer * g.n_q_heads + kvh * G + gq) * g.n_seqs + seq) * D;
  if (n_blk <= 0) {
    if (t < D) dst[t] = 0.f;
    return;
  }
  float m_run = -INFINITY, a = 0.f, l = 0.f;
  for (int b0 = pt; b0 < n_blk; b0 += NP * U) {
    float mb[U], lb[U], vb[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int b = b0 + u * NP;
      const bool in = b < n_blk;
      const float* bp = hp + (int64_t)(in ? b : b0) * bstride;
      mb[u] = in ? bp[D] : -INFINITY;
      lb[u] = bp[D + 1];
      vb[u] = bp[x];
    }
    float m_new = m_run;
#pragma unroll
    for (int u = 0; u < U; ++u) m_new = fmaxf(m_new, mb[u]);     // finite: block b0 holds a row
    const float keep = __expf(m_run - m_new);                    // exp(-inf) = 0 the first time
    a *= keep;
    l *= keep;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float e = __expf(mb[u] - m_new);
      a = fmaf(vb[u], e, a);
      l = fmaf(lb[u], e, l);
    }
    m_run = m_new;
  }
  accs[pt][x] = a;
  if (x == 0) {
    pm[pt] = m_run;
    pl[pt] = l;
  }
  __syncthreads();
  if (t < D) {
    float M = pm[0];
#pragma unroll
    for (int q2 = 1; q2 < NP; ++q2) M = fmaxf(M, pm[q2]);        // group 0 always holds block 0
    float tot = 0.f, den = 0.f;
#pragma unroll
    for (int q2 = 0; q2 < NP; ++q2) {
      const float e = __expf(pm[q2] - M);                        // a group without blocks: exp(-inf) = 0
      tot = fmaf(accs[q2][t], e, tot);
      den = fmaf(pl[q2], e, den);
    }
    dst[t] = tot / den;
  }
}

int decode_rows_per_block(const HostCfg&) { return kDecRows; }

int64_t decode_workspace_bytes(const HostCfg& hc) {
  const int R = decode_rows_per_block(hc);
  const int64_t max_blocks = (hc.max_len + R - 1) / R;
  return (int64_t)hc.n_hi * max_blocks * hc.g.group * (hc.g.head_dim + 2) * 4;
}

template <bool F32, int D, int NG>
static int launch_decode_t(const HostCfg& hc, const void* q, const void* kp, const void* vp,
                           const int64_t* offsets, float* out, char* ws, hipStream_t st) {
  constexpr int R = kDecRows;
  const Geom& g = hc.g;
  DecGeom dg{g.n_layers, g.n_q_heads, g.n_kv_heads, g.group, hc.seq.n_seqs, (hc.max_len + R - 1) / R,
             g.scale_log2e * 0.69314718055994530942f};
  float* part = reinterpret_cast<float*>(ws);
  hipLaunchKernelGGL((decode_partial_kernel<F32, D, NG>), dim3(dg.max_blocks, hc.n_hi, (g.group + NG - 1) / NG),
                     dim3(64 * kDecWaves), 0, st, dg, (const char*)q, (const char*)kp, (const char*)vp, offsets, part);
  hipLaunchKernelGGL((decode_combine_kernel<D, R>), dim3(g.group, hc.n_hi), dim3(1024), 0, st, dg, offsets,
                     (const float*)part, out);
  return check_launch();
}

template <bool F32, int D>
static int launch_decode_g(const HostCfg& hc, const void* q, const void* kp, const void* vp,
                           const int64_t* offsets, float* out, char* ws, hipStream_t st) {
  // four queries at a time for small groups, eight otherwise (larger groups take several passes)
  if (hc.g.group <= 4) return launch_decode_t<F32, D, 4>(hc, q, kp, vp, offsets, out, ws, st);
  return launch_decode_t<F32, D, 8>(hc, q, kp, vp, offsets, out, ws, st);
}

int launch_decode(const HostCfg& hc, const void* q, const void* kp, const void* vp, const int64_t* offsets,
                  float* out, char* ws, hipStream_t st) {
  const Geom& g = hc.g;
  if (g.group > kDecMaxGroup) return LUKV_EINVAL;
  if (!g.f32 && g.head_dim == 128) return launch_decode_g<false, 128>(hc, q, kp, vp, offsets, out, ws, st);
  if (!g.f32 && g.head_dim == 64) return launch_decode_g<false, 64>(hc, q, kp, vp, offsets, out, ws, st);
  if (g.f32 && g.head_dim == 128) return launch_decode_g<true, 128>(hc, q, kp, vp, offsets, out, ws, st);
  if (g.f32 && g.head_dim == 64) return launch_decode_g<true, 64>(hc, q, kp, vp, offsets, out, ws, st);
  return LUKV_EDTYPE;
}

}  // namespace lukv
