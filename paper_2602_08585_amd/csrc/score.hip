// Step 1: observation-window score (Eq. 1 softmax over the cached keys for the last w
// queries; SnapKV metric with kernel pooling, App. D Table 8; always-kept sink / recent
// window, App. E).
//
// Two streaming passes over K per (layer, sequence, KV head):
//   stats  - S = K_tile * Q^T on the matrix cores; every lane owns one query row of a 32x32
//            block and folds its 16 logits into a running (max, sum exp2) pair; the last
//            workgroup of a head merges the per-chunk pairs into one constant per row,
//            c_r = max_r * a + log2(sum_r), a = scale * log2(e).
//   accum  - S = Q * K_tile^T, so that a lane owns one key column; P = exp2(S*a - c_r) is
//            summed over the G*w rows in registers and written as the unpooled metric.
// A third, tiny kernel applies the clipped max-pool and the +inf of forced positions.
//
// Matrix-core operand layout (v_mfma_f32_32x32x16_bf16 / 32x32x2_f32): lane l supplies row
// l%32 of its operand and the k-slice selected by l/32; both operands use the same rule
// "half hf = l/32 owns elements [hf*D/2, (hf+1)*D/2) of the row", so any internal ordering
// of k is the same on both sides.  Output: acc[v] is row 8*(v/4) + 4*(l/32) + v%4, column l%32.
#include "lukv_internal.hpp"

namespace lukv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

template <bool F32>
__device__ __forceinline__ f32x16 mma(uint4 a, uint4 b, f32x16 c) {
  if constexpr (!F32) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  } else {
    f32x4 fa = __builtin_bit_cast(f32x4, a), fb = __builtin_bit_cast(f32x4, b);
#pragma unroll
    for (int e = 0; e < 4; ++e) c = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[e], fb[e], c, 0, 0, 0);
    return c;
  }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <bool F32, int D>
struct Tile {
  static constexpr int kEsize = F32 ? 4 : 2;
  static constexpr int kRowBytes = D * kEsize;
  static constexpr int kRowU4 = kRowBytes / 16;        // 16-byte units per row
  static constexpr int kHalfU4 = kRowU4 / 2;           // units one lane half consumes
  static constexpr int kLdsRowU4 = kRowU4 + 1;         // +16 B pad: conflict-free b128 reads
  static constexpr int kMaxKeys = 128;
};

// Copy `keys` rows of K (sequence-relative rows j0.., clamped to L-1) into LDS.
template <bool F32, int D>
__device__ __forceinline__ void load_k_tile(uint4* lds, const char* kbase, int64_t tok_stride_bytes,
                                            int j0, int keys, int L) {
  using T = Tile<F32, D>;
  const int n = keys * T::kRowU4;
  for (int idx = threadIdx.x; idx < n; idx += 256) {
    const int row = idx / T::kRowU4, col = idx % T::kRowU4;
    int j = j0 + row;
    j = j < L ? j : L - 1;
    const uint4 val = *reinterpret_cast<const uint4*>(kbase + (int64_t)j * tok_stride_bytes + col * 16);
    lds[row * T::kLdsRowU4 + col] = val;
  }
}

// Window-query rows of this wave's row blocks, as matrix-core operands held in registers.
template <bool F32, int D, int NBM, int HU>
__device__ __forceinline__ void load_q(uint4 (&qreg)[NBM][HU], const Geom& g,
                                       const char* q, int layer, int kvh, int seq, int blk0,
                                       int nb_count, int lane) {
  using T = Tile<F32, D>;
  const int hf = lane >> 5;
#pragma unroll
  for (int nb = 0; nb < NBM; ++nb) {
    const int r = 32 * (blk0 + nb) + (lane & 31);
    const bool live = nb < nb_count && r < g.rows;
    const int gq = live ? r / g.window : 0, i = live ? r % g.window : 0;
    const char* p = q + ((int64_t)layer * g.qsl + (int64_t)(kvh * g.group + gq) * g.qsh +
                         (int64_t)(seq * g.window + i) * g.qst) * T::kEsize +
                    hf * (T::kRowBytes / 2);
#pragma unroll
    for (int s = 0; s < T::kHalfU4; ++s)
      qreg[nb][s] = live ? reinterpret_cast<const uint4*>(p)[s] : make_uint4(0, 0, 0, 0);
  }
}

__device__ __forceinline__ void merge_stats(float& m, float& z, float m2, float z2, float a) {
  const float mm = fmaxf(m, m2);
  const float ms = mm == -INFINITY ? 0.f : mm;
  z = z * fast_exp2((m - ms) * a) + z2 * fast_exp2((m2 - ms) * a);
  m = mm;
}

// ---- pass A: softmax statistics ----------------------------------------------------------
template <bool F32, int D, int NBM>
__global__ __launch_bounds__(256) void score_stats_kernel(Geom g, SeqTab tab, const char* q,
                                                          const char* k, float2* partial,
                                                          float* rowc, unsigned* counter,
                                                          int max_chunks, int rows_padded) {
  using T = Tile<F32, D>;
  __shared__ uint4 ktile[T::kMaxKeys * T::kLdsRowU4];
  __shared__ float2 wstat[4][NBM][32];
  __shared__ int is_last;

  int seq, ch;
  find_tile(tab, blockIdx.x, seq, ch);
  const int kvh = blockIdx.y, layer = blockIdx.z;
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0, P = L - g.window;
  const int hi = (seq * g.n_layers + layer) * g.n_kv_heads + kvh;
  const int n_chunks = tab.tile0[seq + 1] - tab.tile0[seq];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5;
  const int n_kt = 4 / g.row_groups, kt = wave % n_kt, rg = wave / n_kt;
  const int keys_per_iter = 32 * n_kt;
  const int blk0 = rg * g.blocks_per_group;
  int nb_count = g.row_blocks - blk0;
  nb_count = nb_count < 0 ? 0 : (nb_count > g.blocks_per_group ? g.blocks_per_group : nb_count);
  const float a = g.scale_log2e;

  uint4 qreg[NBM][T::kHalfU4];
  load_q<F32, D, NBM, T::kHalfU4>(qreg, g, q, layer, kvh, seq, blk0, nb_count, lane);

  // window row index of this lane's query in every block (for the causal range)
  int wrow[NBM];
#pragma unroll
  for (int nb = 0; nb < NBM; ++nb) wrow[nb] = (32 * (blk0 + nb) + (lane & 31)) % g.window;

  float m[NBM], z[NBM];
#pragma unroll
  for (int nb = 0; nb < NBM; ++nb) { m[nb] = -INFINITY; z[nb] = 0.f; }

  const char* kbase = k + ((int64_t)layer * g.sl + (int64_t)kvh * g.sh + (int64_t)tok0 * g.st) * T::kEsize;
  const int64_t tok_bytes = g.st * T::kEsize;
  const int j_begin = ch * kChunkKeys;
  const int j_end = min(L, j_begin + kChunkKeys);

  for (int j0 = j_begin; j0 < j_end; j0 += keys_per_iter) {
    __syncthreads();
    load_k_tile<F32, D>(ktile, kbase, tok_bytes, j0, keys_per_iter, L);
    __syncthreads();
    const int jw = j0 + 32 * kt;           // first key of this wave's 32-key subtile
    if (jw >= j_end) continue;             // uniform per wave; barriers above are unconditional
    uint4 kreg[T::kHalfU4];
    const uint4* src = ktile + (32 * kt + (lane & 31)) * T::kLdsRowU4 + hf * T::kHalfU4;
#pragma unroll
    for (int s = 0; s < T::kHalfU4; ++s) kreg[s] = src[s];
    const bool need_mask = jw + 32 > P;
#pragma unroll
    for (int nb = 0; nb < NBM; ++nb) {
      if (nb < nb_count) {
        f32x16 acc = {0};
#pragma unroll
        for (int s = 0; s < T::kHalfU4; ++s) acc = mma<F32>(kreg[s], qreg[nb][s], acc);
        if (need_mask) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int j = jw + 8 * (v >> 2) + 4 * hf + (v & 3);
            if (j >= L || j > P + wrow[nb]) acc[v] = -INFINITY;
          }
        }
        float tm = acc[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) tm = fmaxf(tm, acc[v]);
        const float mn = fmaxf(m[nb], tm);
        const float ms = mn == -INFINITY ? 0.f : mn;
        float zz = z[nb] * fast_exp2((m[nb] - ms) * a);
        const float off = -ms * a;
#pragma unroll
        for (int v = 0; v < 16; ++v) zz += fast_exp2(fmaf(acc[v], a, off));
        z[nb] = zz;
        m[nb] = mn;
      }
    }
  }

  // lane l and l^32 hold the same query rows over different keys
#pragma unroll
  for (int nb = 0; nb < NBM; ++nb) {
    const float m2 = __shfl_xor(m[nb], 32), z2 = __shfl_xor(z[nb], 32);
    merge_stats(m[nb], z[nb], m2, z2, a);
    if (lane < 32) wstat[wave][nb][lane] = make_float2(m[nb], z[nb]);
  }
  __syncthreads();
  // merge the key subtiles of every row group and publish this chunk's pair per row
  for (int r = threadIdx.x; r < rows_padded; r += 256) {
    const int blk = r >> 5, grp = blk / g.blocks_per_group, nb = blk - grp * g.blocks_per_group;
    float mm = -INFINITY, zz = 0.f;
    if (grp < g.row_groups) {
      for (int t = 0; t < n_kt; ++t) {
        const float2 st = wstat[grp * n_kt + t][nb][r & 31];
        merge_stats(mm, zz, st.x, st.y, a);
      }
    }
    partial[((int64_t)hi * max_chunks + ch) * rows_padded + r] = make_float2(mm, zz);
  }
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) is_last = atomicAdd(&counter[hi], 1u) == (unsigned)(n_chunks - 1);
  __syncthreads();
  if (!is_last) return;
  __threadfence();
  for (int r = threadIdx.x; r < rows_padded; r += 256) {
    float mm = -INFINITY, zz = 0.f;
    for (int c2 = 0; c2 < n_chunks; ++c2) {
      const float* pp = reinterpret_cast<const float*>(&partial[((int64_t)hi * max_chunks + c2) * rows_padded + r]);
      merge_stats(mm, zz, __builtin_nontemporal_load(pp), __builtin_nontemporal_load(pp + 1), a);
    }
    // padded rows never contribute: +inf makes exp2(S*a - c) vanish in pass B
    rowc[(int64_t)hi * rows_padded + r] = r < g.rows ? mm * a + log2f(zz) : INFINITY;
  }
}

// ---- pass B: normalised window sums ------------------------------------------------------
template <bool F32, int D, int NBM>
__global__ __launch_bounds__(256) void score_accum_kernel(Geom g, SeqTab tab, const char* q,
                                                          const char* k, const float* rowc,
                                                          float* raw, int rows_padded) {
  using T = Tile<F32, D>;
  __shared__ uint4 ktile[T::kMaxKeys * T::kLdsRowU4];
  __shared__ __align__(16) float rowc_s[kMaxRows];
  __shared__ float colred[4][32];

  int seq, ch;
  find_tile(tab, blockIdx.x, seq, ch);
  const int kvh = blockIdx.y, layer = blockIdx.z;
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0, P = L - g.window;
  const int hi = (seq * g.n_layers + layer) * g.n_kv_heads + kvh;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, hf = lane >> 5;
  const int n_kt = 4 / g.row_groups, kt = wave % n_kt, rg = wave / n_kt;
  const int keys_per_iter = 32 * n_kt;
  const int blk0 = rg * g.blocks_per_group;
  int nb_count = g.row_blocks - blk0;
  nb_count = nb_count < 0 ? 0 : (nb_count > g.blocks_per_group ? g.blocks_per_group : nb_count);
  const float a = g.scale_log2e;

  for (int r = threadIdx.x; r < kMaxRows; r += 256)
    rowc_s[r] = r < rows_padded ? rowc[(int64_t)hi * rows_padded + r] : INFINITY;

  uint4 qreg[NBM][T::kHalfU4];
  load_q<F32, D, NBM, T::kHalfU4>(qreg, g, q, layer, kvh, seq, blk0, nb_count, lane);

  const char* kbase = k + ((int64_t)layer * g.sl + (int64_t)kvh * g.sh + (int64_t)tok0 * g.st) * T::kEsize;
  const int64_t tok_bytes = g.st * T::kEsize;
  float* out = raw + ((int64_t)layer * g.n_kv_heads + kvh) * g.total_tokens + tok0;
  const int j_begin = ch * kChunkKeys;
  const int j_end = min(P, j_begin + kChunkKeys);

  for (int j0 = j_begin; j0 < j_end; j0 += keys_per_iter) {
    __syncthreads();
    load_k_tile<F32, D>(ktile, kbase, tok_bytes, j0, keys_per_iter, L);
    __syncthreads();
    const int jw = j0 + 32 * kt;
    float col = 0.f;
    if (jw < j_end) {
      uint4 kreg[T::kHalfU4];
      const uint4* src = ktile + (32 * kt + (lane & 31)) * T::kLdsRowU4 + hf * T::kHalfU4;
#pragma unroll
      for (int s = 0; s < T::kHalfU4; ++s) kreg[s] = src[s];
#pragma unroll
      for (int nb = 0; nb < NBM; ++nb) {
        if (nb < nb_count) {
          f32x16 acc = {0};
#pragma unroll
          for (int s = 0; s < T::kHalfU4; ++s) acc = mma<F32>(qreg[nb][s], kreg[s], acc);
          const float* rc = rowc_s + 32 * (blk0 + nb) + 4 * hf;
#pragma unroll
          for (int v4 = 0; v4 < 4; ++v4) {
            const f32x4 c4 = *reinterpret_cast<const f32x4*>(rc + 8 * v4);
#pragma unroll
            for (int e = 0; e < 4; ++e) col += fast_exp2(fmaf(acc[4 * v4 + e], a, -c4[e]));
          }
        }
      }
      col += __shfl_xor(col, 32);
    }
    if (g.row_groups > 1) {
      // fixed-order sum over the row groups keeps the result deterministic
      if (lane < 32) colred[wave][lane] = col;
      __syncthreads();
      if (rg == 0) {
        for (int t = 1; t < g.row_groups; ++t) col += colred[t * n_kt + kt][lane & 31];
      }
    }
    if (rg == 0 && lane < 32 && jw + lane < j_end) out[jw + lane] = col * g.inv_group;
  }
}

// ---- pooling + forced positions ----------------------------------------------------------
__global__ __launch_bounds__(256) void pool_kernel(Geom g, SeqTab tab, const float* raw,
                                                   float* pooled) {
  int seq, tile;
  find_tile(tab, blockIdx.x, seq, tile);
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0, P = L - g.window;
  const int j = tile * 256 + threadIdx.x;
  if (j >= L) return;
  const int64_t base = (int64_t)blockIdx.y * g.total_tokens + tok0;
  float s = INFINITY;
  if (j >= g.n_sink && j < P) {
    const int h = g.pool_kernel >> 1;
    const int lo = max(0, j - h), hi = min(P - 1, j + h);
    s = raw[base + lo];
    for (int t = lo + 1; t <= hi; ++t) s = fmaxf(s, raw[base + t]);
  }
  pooled[base + j] = s;
}

// ---- launcher ----------------------------------------------------------------------------
template <bool F32, int D, int NBM>
static int launch_score_t(const HostCfg& hc, const WsLayout& lay, const void* q, const void* k,
                          float* pooled_out, char* ws, hipStream_t st) {
  const Geom& g = hc.g;
  float2* partial = reinterpret_cast<float2*>(ws + lay.partial);
  float* rowc = reinterpret_cast<float*>(ws + lay.rowc);
  float* raw = reinterpret_cast<float*>(ws + lay.raw);
  unsigned* cnt = reinterpret_cast<unsigned*>(ws + lay.stats_cnt);
  const SeqTab tabA = tiles_for(hc.seq, kChunkKeys, 0);
  const SeqTab tabB = tiles_for(hc.seq, kChunkKeys, g.window);
  const SeqTab tabP = tiles_for(hc.seq, 256, 0);
  dim3 gridA(tabA.tile0[tabA.n_seqs], g.n_kv_heads, g.n_layers);
  dim3 gridB(tabB.tile0[tabB.n_seqs], g.n_kv_heads, g.n_layers);
  dim3 gridP(tabP.tile0[tabP.n_seqs], g.n_kv_heads * g.n_layers, 1);
  stage_mark(kStStats, st);
  hipLaunchKernelGGL((score_stats_kernel<F32, D, NBM>), gridA, dim3(256), 0, st, g, tabA,
                     (const char*)q, (const char*)k, partial, rowc, cnt, lay.max_chunks,
                     lay.rows_padded);
  stage_mark(kStAccum, st);
  hipLaunchKernelGGL((score_accum_kernel<F32, D, NBM>), gridB, dim3(256), 0, st, g, tabB,
                     (const char*)q, (const char*)k, (const float*)rowc, raw, lay.rows_padded);
  stage_mark(kStPool, st);
  hipLaunchKernelGGL(pool_kernel, gridP, dim3(256), 0, st, g, tabP, (const float*)raw, pooled_out);
  return check_launch();
}

int launch_score(const HostCfg& hc, const WsLayout& lay, const void* q, const void* k,
                 float* pooled_out, char* ws, hipStream_t st) {
  const Geom& g = hc.g;
  if (!g.f32 && g.head_dim == 128) return launch_score_t<false, 128, 4>(hc, lay, q, k, pooled_out, ws, st);
  if (!g.f32 && g.head_dim == 64) return launch_score_t<false, 64, 4>(hc, lay, q, k, pooled_out, ws, st);
  if (g.f32 && g.head_dim == 64) return launch_score_t<true, 64, 4>(hc, lay, q, k, pooled_out, ws, st);
  if (g.f32 && g.head_dim == 128) return launch_score_t<true, 128, 2>(hc, lay, q, k, pooled_out, ws, st);
  return LUKV_EDTYPE;
}

}  // namespace lukv
