// Consumer of the compacted cache: one decode step's attention over the retained entries of
// every head (Sec. 3.2, Eq. 3 restricted to the index set I_{l,h}).  The packed K and V rows of
// head hi sit at [offsets[hi], offsets[hi+1]); the G query heads of a group share them.
//   decode_partial - one workgroup per (head, block of 128 rows): K tile through LDS, the G logits
//                    of every row on the matrix cores (bf16; plain dot products for f32), block
//                    softmax statistics, then the V tile through the same LDS buffer and
//                    p-weighted column sums; leaves (max, sum, weighted values) per query head.
//   decode_combine - one workgroup per (query head, head): merges the blocks' partial results.
// Row counts live on the device (they are budgets), so the grid covers the longest possible
// head and workgroups beyond a head's rows exit at once.
#include "lukv_internal.hpp"

namespace lukv {

constexpr int kDecMaxGroup = 16;   // query heads per KV head the decode kernels take

struct DecGeom {
  int32_t n_layers, n_q_heads, n_kv_heads, group, n_seqs, max_blocks;
  float scale;
};

// R rows per block; a row is D elements = kRowU4 16-byte pieces, padded by one piece in LDS.
template <bool F32, int D, int R>
__global__ __launch_bounds__(256) void decode_partial_kernel(DecGeom g, const char* q, const char* kp,
                                                             const char* vp, const int64_t* offsets,
                                                             float* part) {
  constexpr int kEsize = F32 ? 4 : 2;
  constexpr int kRowU4 = D * kEsize / 16;
  constexpr int kLdsRowU4 = kRowU4 + 1;
  constexpr int kLoads = R * kRowU4 / 256;
  constexpr int kPerU4 = 16 / kEsize;            // elements in one 16-byte piece
  __shared__ u32x4 tile[R * kLdsRowU4];
  __shared__ u32x4 qbuf[32 * kLdsRowU4];          // the group's queries: 32 padded rows (bf16) or floats
  __shared__ float ps[kDecMaxGroup * R];
  __shared__ float red[4][kDecMaxGroup];
  __shared__ float stat[2][kDecMaxGroup];
  const int hi = blockIdx.y, blk = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t row_begin = offsets[hi] + (int64_t)blk * R;
  const int64_t rows_left = offsets[hi + 1] - row_begin;
  if (rows_left <= 0) return;
  const int n = rows_left < R ? (int)rows_left : R;
  const int G = g.group;
  const int kvh = hi % g.n_kv_heads, layer = (hi / g.n_kv_heads) % g.n_layers;
  const int seq = hi / (g.n_kv_heads * g.n_layers);
  static_assert(R == 128, "four waves of 32 rows / two threads per row");

  // K and V tiles: 16 bytes per lane, rows beyond the block clamped to its last row
  u32x4 kr[kLoads], vr[kLoads];
#pragma unroll
  for (int u = 0; u < kLoads; ++u) {
    const int i = u * 256 + t, r = i / kRowU4, c = i % kRowU4;
    const int64_t row = row_begin + (r < n ? r : n - 1);
    kr[u] = *reinterpret_cast<const u32x4*>(kp + (row * kRowU4 + c) * 16);
    vr[u] = *reinterpret_cast<const u32x4*>(vp + (row * kRowU4 + c) * 16);
  }
  auto q_row = [&](int gq) {   // element index of query head gq's row
    return (((int64_t)layer * g.n_q_heads + kvh * G + gq) * g.n_seqs + seq) * D;
  };
  float* qs = reinterpret_cast<float*>(qbuf);
  if constexpr (F32) {
    // the group's decode queries as floats
    for (int i = t; i < G * D; i += 256) qs[i] = reinterpret_cast<const float*>(q)[q_row(i / D) + i % D];
  } else {
    // as a 32-row bf16 operand tile (rows beyond the group are zero)
    for (int i = t; i < 32 * kRowU4; i += 256) {
      const int r = i / kRowU4, c = i % kRowU4;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (r < G) v = *reinterpret_cast<const u32x4*>(q + (q_row(r) + c * 8) * 2);
      qbuf[r * kLdsRowU4 + c] = v;
    }
  }
#pragma unroll
  for (int u = 0; u < kLoads; ++u) {
    const int i = u * 256 + t;
    tile[(i / kRowU4) * kLdsRowU4 + i % kRowU4] = kr[u];
  }
  __syncthreads();

  auto fmax_bits = [](unsigned x, unsigned y) { return __float_as_uint(fmaxf(__uint_as_float(x), __uint_as_float(y))); };
  auto fadd_bits = [](unsigned x, unsigned y) { return __float_as_uint(__uint_as_float(x) + __uint_as_float(y)); };
  if constexpr (!F32) {
    // logits on the matrix cores: wave w takes rows 32w .. 32w+31, S = K_rows * Q^T (32 x 32, the
    // first G columns live).  Both operands: lane l supplies row l%32 and, of its half l/32 of
    // the row, the 8 elements of step s.  acc[v] is row 8*(v/4) + 4*(l/32) + v%4, column l%32.
    typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
    typedef __attribute__((ext_vector_type(16))) float f32x16;
    const int hf = lane >> 5, gq = lane & 31;
    f32x16 acc = {0};
#pragma unroll
    for (int st = 0; st < kRowU4 / 2; ++st) {
      const u32x4 av = tile[(32 * wave + gq) * kLdsRowU4 + hf * (kRowU4 / 2) + st];
      const u32x4 bv = qbuf[gq * kLdsRowU4 + hf * (kRowU4 / 2) + st];
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bv),
                                                    acc, 0, 0, 0);
    }
    float sv[16], m = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = 32 * wave + 8 * (v >> 2) + 4 * hf + (v & 3);
      sv[v] = r < n ? acc[v] * g.scale : -INFINITY;
      m = fmaxf(m, sv[v]);
    }
    m = fmaxf(m, __shfl_xor(m, 32));                 // the two halves of the rows
    if (lane < 32 && gq < G) red[wave][gq] = m;
    __syncthreads();
    if (t < G) stat[0][t] = fmaxf(fmaxf(red[0][t], red[1][t]), fmaxf(red[2][t], red[3][t]));
    __syncthreads();
    const float M = gq < G ? stat[0][gq] : 0.f;
    float l = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = 32 * wave + 8 * (v >> 2) + 4 * hf + (v & 3);
      const float pv = r < n ? __expf(sv[v] - M) : 0.f;
      if (gq < G) ps[gq * R + r] = pv;
      l += pv;
    }
    l += __shfl_xor(l, 32);
    if (lane < 32 && gq < G) red[wave][gq] = l;
  } else {
    // logits: two threads per row, each over half of the row's 16-byte pieces; the upper half's
    // sums pass through LDS
    const int row = t & (R - 1), half = t >> 7;
    float s[kDecMaxGroup];
#pragma unroll
    for (int gq = 0; gq < kDecMaxGroup; ++gq) s[gq] = 0.f;
#pragma unroll 4
    for (int c = half * (kRowU4 / 2); c < (half + 1) * (kRowU4 / 2); ++c) {
      const u32x4 kv = tile[row * kLdsRowU4 + c];
      float kf[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) kf[e] = __uint_as_float(kv[e]);
#pragma unroll
      for (int gq = 0; gq < kDecMaxGroup; ++gq) {
        if (gq < G) {
          const float* qv = qs + gq * D + c * kPerU4;
#pragma unroll
          for (int e = 0; e < kPerU4; ++e) s[gq] = fmaf(qv[e], kf[e], s[gq]);
        }
      }
    }
    if (half) {
#pragma unroll
      for (int gq = 0; gq < kDecMaxGroup; ++gq)
        if (gq < G) ps[gq * R + row] = s[gq];
    }
    __syncthreads();
    if (!half) {
#pragma unroll
      for (int gq = 0; gq < kDecMaxGroup; ++gq)
        if (gq < G) s[gq] += ps[gq * R + row];
    }
    __syncthreads();   // ps is rewritten with the probabilities below
    const bool live = !half && row < n;
    // block maximum and sum of exponentials per query head (wave reductions on DPP steps)
#pragma unroll
    for (int gq = 0; gq < kDecMaxGroup; ++gq) {
      if (gq < G) {
        float m = live ? s[gq] * g.scale : -INFINITY;
        s[gq] = m;
        m = __uint_as_float(wave_reduce_to_last(__float_as_uint(m), 0xFF800000u, fmax_bits));
        if (lane == 63) red[wave][gq] = m;
      }
    }
    __syncthreads();
    if (t < G) stat[0][t] = fmaxf(fmaxf(red[0][t], red[1][t]), fmaxf(red[2][t], red[3][t]));
    __syncthreads();
#pragma unroll
    for (int gq = 0; gq < kDecMaxGroup; ++gq) {
      if (gq < G) {
        const float p = live ? __expf(s[gq] - stat[0][gq]) : 0.f;
        if (t < R) ps[gq * R + t] = p;
        const float l = __uint_as_float(wave_reduce_to_last(__float_as_uint(p), 0u, fadd_bits));
        if (lane == 63) red[wave][gq] = l;
      }
    }
  }
  // the V tile takes the K tile's place (every thread is done reading K)
  __syncthreads();
  if (t < G) stat[1][t] = (red[0][t] + red[1][t]) + (red[2][t] + red[3][t]);
#pragma unroll
  for (int u = 0; u < kLoads; ++u) {
    const int i = u * 256 + t;
    tile[(i / kRowU4) * kLdsRowU4 + i % kRowU4] = vr[u];
  }
  __syncthreads();

  // p-weighted column sums: one (query head, pair of columns) at a time per thread
  float* my_part = part + ((int64_t)hi * g.max_blocks + blk) * G * (D + 2);
  const unsigned* tile32 = reinterpret_cast<const unsigned*>(tile);
  constexpr int kCols = F32 ? 1 : 2;             // columns in one 32-bit word
  constexpr int kWords = D / kCols;
  for (int o = t; o < G * kWords; o += 256) {
    const int gq = o / kWords, wd = o - gq * kWords;
    const float* pg = ps + gq * R;
    float a0 = 0.f, a1 = 0.f;
    // rows beyond n carry p = 0 and a valid (clamped) row, so the loop runs over the whole
    // block in steps of eight with the LDS reads of a step in flight together
    for (int r0 = 0; r0 < R; r0 += 8) {
      unsigned w[8];
      float p[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) { w[u] = tile32[(r0 + u) * (kLdsRowU4 * 4) + wd]; p[u] = pg[r0 + u]; }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if constexpr (F32) {
          a0 = fmaf(p[u], __uint_as_float(w[u]), a0);
        } else {
          a0 = fmaf(p[u], __uint_as_float(w[u] << 16), a0);
          a1 = fmaf(p[u], __uint_as_float(w[u] & 0xFFFF0000u), a1);
        }
      }
      if (r0 + 8 >= n) break;
    }
    my_part[gq * (D + 2) + wd * kCols] = a0;
    if constexpr (!F32) my_part[gq * (D + 2) + wd * kCols + 1] = a1;
  }
  if (t < G) {
    my_part[t * (D + 2) + D] = stat[0][t];
    my_part[t * (D + 2) + D + 1] = stat[1][t];
  }
}

// One workgroup per (query head of the group, head): the blocks' partial results are merged with
// weights exp(m_b - M); D threads own the columns, 256 / D groups of them share the blocks.
template <int D, int R>
__global__ __launch_bounds__(1024) void decode_combine_kernel(DecGeom g, const int64_t* offsets, const float* part,
                                                              float* out) {
  constexpr int NP = 1024 / D;          // groups of D threads that share the blocks
  __shared__ float red[16];
  __shared__ float wts[1024];
  __shared__ float accs[NP][D];
  const int gq = blockIdx.x, hi = blockIdx.y, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int G = g.group;
  const int kvh = hi % g.n_kv_heads, layer = (hi / g.n_kv_heads) % g.n_layers;
  const int seq = hi / (g.n_kv_heads * g.n_layers);
  const int64_t rows = offsets[hi + 1] - offsets[hi];
  const int n_blk = (int)((rows + R - 1) / R);
  const float* hp = part + ((int64_t)hi * g.max_blocks * G + gq) * (D + 2);
  const int64_t bstride = (int64_t)G * (D + 2);
  const int x = t % D, pt = t / D;
  float* dst = out + (((int64_t)layer * g.n_q_heads + kvh * G + gq) * g.n_seqs + seq) * D;
  if (n_blk == 0) {
    if (t < D) dst[t] = 0.f;
    return;
  }
  auto fmax_bits = [](unsigned a, unsigned b) { return __float_as_uint(fmaxf(__uint_as_float(a), __uint_as_float(b))); };
  auto fadd_bits = [](unsigned a, unsigned b) { return __float_as_uint(__uint_as_float(a) + __uint_as_float(b)); };
  float m = -INFINITY;
  for (int b = t; b < n_blk; b += 1024) m = fmaxf(m, hp[b * bstride + D]);
  m = __uint_as_float(wave_reduce_to_last(__float_as_uint(m), 0xFF800000u, fmax_bits));
  if (lane == 63) red[wave] = m;
  __syncthreads();
  float M = red[0];
#pragma unroll
  for (int w = 1; w < 16; ++w) M = fmaxf(M, red[w]);
  float l = 0.f, a = 0.f;
  for (int b0 = 0; b0 < n_blk; b0 += 1024) {
    __syncthreads();
    float e = 0.f;
    if (b0 + t < n_blk) {
      e = __expf(hp[(b0 + t) * bstride + D] - M);
      l += hp[(b0 + t) * bstride + D + 1] * e;
    }
    wts[t] = e;
    __syncthreads();
    const int nb = n_blk - b0 < 1024 ? n_blk - b0 : 1024;
#pragma unroll 4
    for (int bb = pt; bb < nb; bb += NP) a = fmaf(hp[(b0 + bb) * bstride + x], wts[bb], a);
  }
  l = __uint_as_float(wave_reduce_to_last(__float_as_uint(l), 0u, fadd_bits));
  __syncthreads();
  if (lane == 63) red[wave] = l;
  accs[pt][x] = a;
  __syncthreads();
  if (t < D) {
    float tot = 0.f, den = 0.f;
#pragma unroll
    for (int q2 = 0; q2 < NP; ++q2) tot += accs[q2][t];
#pragma unroll
    for (int w = 0; w < 16; ++w) den += red[w];
    dst[t] = tot / den;
  }
}

int decode_rows_per_block(const HostCfg&) { return 128; }

int64_t decode_workspace_bytes(const HostCfg& hc) {
  const int R = decode_rows_per_block(hc);
  const int64_t max_blocks = (hc.max_len + R - 1) / R;
  return (int64_t)hc.n_hi * max_blocks * hc.g.group * (hc.g.head_dim + 2) * 4;
}

template <bool F32, int D, int R>
static int launch_decode_t(const HostCfg& hc, const void* q, const void* kp, const void* vp,
                           const int64_t* offsets, float* out, char* ws, hipStream_t st) {
  const Geom& g = hc.g;
  DecGeom dg{g.n_layers, g.n_q_heads, g.n_kv_heads, g.group, hc.seq.n_seqs, (hc.max_len + R - 1) / R,
             g.scale_log2e * 0.69314718055994530942f};
  float* part = reinterpret_cast<float*>(ws);
  hipLaunchKernelGGL((decode_partial_kernel<F32, D, R>), dim3(dg.max_blocks, hc.n_hi), dim3(256), 0, st, dg,
                     (const char*)q, (const char*)kp, (const char*)vp, offsets, part);
  hipLaunchKernelGGL((decode_combine_kernel<D, R>), dim3(g.group, hc.n_hi), dim3(1024), 0, st, dg, offsets,
                     (const float*)part, out);
  return check_launch();
}

int launch_decode(const HostCfg& hc, const void* q, const void* kp, const void* vp, const int64_t* offsets,
                  float* out, char* ws, hipStream_t st) {
  const Geom& g = hc.g;
  if (g.group > kDecMaxGroup) return LUKV_EINVAL;
  if (!g.f32 && g.head_dim == 128) return launch_decode_t<false, 128, 128>(hc, q, kp, vp, offsets, out, ws, st);
  if (!g.f32 && g.head_dim == 64) return launch_decode_t<false, 64, 128>(hc, q, kp, vp, offsets, out, ws, st);
  if (g.f32 && g.head_dim == 128) return launch_decode_t<true, 128, 128>(hc, q, kp, vp, offsets, out, ws, st);
  if (g.f32 && g.head_dim == 64) return launch_decode_t<true, 64, 128>(hc, q, kp, vp, offsets, out, ws, st);
  return LUKV_EDTYPE;
}

}  // namespace lukv
