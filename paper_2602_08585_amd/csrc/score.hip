// Step 1: observation-window score (Eq. 1 softmax over the cached keys for the last w
// queries; SnapKV metric with kernel pooling, App. D Table 8; always-kept sink / recent
// window, App. E).
//
// Two streaming passes over K per (layer, sequence, KV head):
//   stats  - S = K_tile * Q^T on the matrix cores; every lane owns one query row of a 32x32
//            block and folds its 16 logits into a running (max, sum exp2) pair; per granule of
//            keys the workgroup leaves one float per row, l = max * a + log2(sum),
//            a = scale * log2(e).  A granule is 512 keys, doubled until the sequence has at most
//            64 of them: it depends on the sequence length only, a workgroup's chunk is a whole
//            number of granules, and the merge below runs over granules in index order - so a
//            score does not depend on how a call is cut into workgroups.
//   accum  - merges the head's granule values into one constant per row, c_r = M + log2(sum
//            exp2(l - M)), M = max l (or takes the caller's log-sum-exp); then
//            S = Q * K_tile^T, so that a lane owns one key column; P = exp2(S*a - c_r) is
//            summed over the G*w rows in registers and written as the unpooled metric,
//            together with the (min, max) of what each wave wrote.
// A third, tiny kernel applies the clipped max-pool and the +inf of forced positions when
// the scores are wanted on their own (lukv_score); the fused path pools inside selection.
//
// A workgroup (4 waves) streams a chunk of 512 to 2048 keys in tiles of 128/RG keys: the next tile is
// in flight from HBM into registers while the current one, staged in LDS with a 16-byte row
// pad (conflict-free 128-bit reads), feeds the matrix cores.  RG wave groups share the row
// blocks when G*w > 32*NBM.
//
// Matrix-core operand layout (v_mfma_f32_32x32x16_bf16 / 32x32x2_f32): lane l supplies row
// l%32 of its operand and the k-slice selected by l/32; both operands use the same rule
// "half hf = l/32 owns elements [hf*D/2, (hf+1)*D/2) of the row", so any internal ordering
// of k is the same on both sides.  Output: acc[v] is row 8*(v/4) + 4*(l/32) + v%4, column l%32.
//
// When the fused path asks for it, the hull vertices of the budget allocation (which does not
// depend on scores) are computed along the way: one knot per wave in the workgroups' prologues,
// or, in calls with few workgroups, by a few extra workgroups at the front of the grid.
#include <string.h>

#include <type_traits>

#include "alloc_device.hpp"
#include "lukv_internal.hpp"


namespace lukv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

template <bool F32>
__device__ __forceinline__ f32x16 mma(u32x4 a, u32x4 b, f32x16 c) {
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

// Orders the LDS traffic of one wave (its LDS operations execute in order; this keeps the
// compiler from moving them across) without involving the other waves of the workgroup.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

template <bool PRIVATE>
__device__ __forceinline__ void tile_sync() {
  if constexpr (PRIVATE) wave_sync(); else __syncthreads();
}

template <bool F32, int D, int RG>
struct Tile {
  static constexpr int kEsize = F32 ? 4 : 2;
  static constexpr int kRowBytes = D * kEsize;
  static constexpr int kRowU4 = kRowBytes / 16;        // 16-byte units per row
  static constexpr int kHalfU4 = kRowU4 / 2;           // units one lane half consumes
  static constexpr int kLdsRowU4 = kRowU4 + 1;         // +16 B pad: conflict-free b128 reads
  static constexpr int kKeys = 128 / RG;               // keys per tile
  static constexpr int kWaveCols = 4 / RG;             // 32-key subtiles per tile
  static constexpr int kLoads = kKeys * kRowU4 / 256;  // 16-byte loads per thread per tile
  // With one row group every wave consumes only its own 32 keys of a tile, so it also loads
  // them itself (64 lanes cover 64/kRowU4 rows per load) and never waits for the other waves;
  // with several row groups the 256 threads load the shared tile together.
  static constexpr bool kPrivate = RG == 1;
  static constexpr int kLoadRowStep = (kPrivate ? 64 : 256) / kRowU4;   // rows between a thread's loads
  static_assert(kLoads >= 1, "tile too small for 256 threads");
  static_assert(!kPrivate || kLoads * kLoadRowStep == 32, "a wave loads exactly its 32 keys");
};

// One thread's share of a K tile (plain local arrays: they must stay in registers so that
// the loads of the next tile are in flight while the current one is consumed).
// k_issue starts the loads (rows clamped to L-1), k_commit stores them to LDS.
// `off0` is this thread's byte offset (from the head's first key) of its first row of the
// tile; the other rows follow at a uniform stride; rows past the sequence clamp to the last.
template <bool F32, int D, int RG, int NL>
__device__ __forceinline__ void k_issue(u32x4 (&pre)[NL], const char* kbase, unsigned off0,
                                        unsigned row_stride_bytes, unsigned off_last) {
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    unsigned off = off0 + (unsigned)i * row_stride_bytes;
    off = off < off_last ? off : off_last;
    pre[i] = *reinterpret_cast<const u32x4*>(kbase + off);
  }
}

template <bool F32, int D, int RG, int NL>
__device__ __forceinline__ void k_commit(const u32x4 (&pre)[NL], u32x4* lds, int lds_off) {
  using T = Tile<F32, D, RG>;
#pragma unroll
  for (int i = 0; i < NL; ++i) lds[lds_off + i * T::kLoadRowStep * T::kLdsRowU4] = pre[i];
}

// Window-query rows of this wave's row blocks, as matrix-core operands held in registers.
// The workgroup fetches the rows of one row group at a time with coalesced loads (q_fetch),
// parks them in the K-tile buffer (q_park) and every wave of that group picks its operand
// layout from there (q_pick): one L2 read per workgroup instead of one per wave.
template <bool F32, int D, int NBM>
struct QStage {
  static constexpr int kEsize = F32 ? 4 : 2;
  static constexpr int kRowU4 = D * kEsize / 16;
  static constexpr int kLdsRowU4 = kRowU4 + 1;
  static constexpr int kRows = 32 * NBM;                 // rows of one row group
  static constexpr int kLoads = kRows * kRowU4 / 256;    // 16-byte loads per thread
  static constexpr int kRowStep = 256 / kRowU4;
};

template <bool F32, int D, int NBM, int NQ>
__device__ __forceinline__ void q_fetch(u32x4 (&tmp)[NQ], const Geom& g,
                                        const char* q, int layer, int kvh, int seq, int group) {
  using QS = QStage<F32, D, NBM>;
  const int row0 = threadIdx.x / QS::kRowU4, col = threadIdx.x % QS::kRowU4;
#pragma unroll
  for (int i = 0; i < QS::kLoads; ++i) {
    const int lr = row0 + i * QS::kRowStep;                       // row inside the group
    const int r = 32 * group * g.blocks_per_group + lr;           // row of the head
    const bool live = lr < 32 * g.blocks_per_group && r < g.rows;
    const int gq = live ? r / g.window : 0, wi = live ? r % g.window : 0;
    const char* p = q + ((int64_t)layer * g.qsl + (int64_t)(kvh * g.group + gq) * g.qsh +
                         (int64_t)(seq * g.window + wi) * g.qst) * QS::kEsize + col * 16;
    tmp[i] = live ? *reinterpret_cast<const u32x4*>(p) : u32x4{0u, 0u, 0u, 0u};
  }
}

template <bool F32, int D, int NBM, int NQ>
__device__ __forceinline__ void q_park(const u32x4 (&tmp)[NQ], u32x4* lds) {
  using QS = QStage<F32, D, NBM>;
  const int row0 = threadIdx.x / QS::kRowU4, col = threadIdx.x % QS::kRowU4;
#pragma unroll
  for (int i = 0; i < QS::kLoads; ++i) lds[(row0 + i * QS::kRowStep) * QS::kLdsRowU4 + col] = tmp[i];
}

template <bool F32, int D, int NBM, int HU>
__device__ __forceinline__ void q_pick(u32x4 (&qreg)[NBM][HU], const u32x4* lds, int lane) {
  using QS = QStage<F32, D, NBM>;
  const int hf = lane >> 5;
#pragma unroll
  for (int nb = 0; nb < NBM; ++nb)
#pragma unroll
    for (int s = 0; s < QS::kRowU4 / 2; ++s)
      qreg[nb][s] = lds[(32 * nb + (lane & 31)) * QS::kLdsRowU4 + hf * (QS::kRowU4 / 2) + s];
}

__device__ __forceinline__ void merge_stats(float& m, float& z, float m2, float z2, float a) {
  const float mm = fmaxf(m, m2);
  const float ms = mm == -INFINITY ? 0.f : mm;
  z = z * fast_exp2((m - ms) * a) + z2 * fast_exp2((m2 - ms) * a);
  m = mm;
}

// Keys per granule of softmax statistics for a sequence of L keys: 512, doubled until there are
// at most kMaxGranules granules.  Chunks of keys (what a workgroup streams) are multiples of it.
constexpr int kMaxGranules = 64;
__host__ __device__ inline int granule_keys(int L) {
  int gkeys = 512;
  while ((L + gkeys - 1) / gkeys > kMaxGranules) gkeys *= 2;
  return gkeys;
}

// Knot of the allocation's first phase that this wave takes in the spread form (-1: none).
// Scoring workgroups are numbered over the whole grid; workgroup b owns knots [b*kp, (b+1)*kp),
// one per wave.
__device__ __forceinline__ int64_t spread_item(const AllocIO& aio, int kp, int n_front_blocks) {
  if (kp <= 0) return -1;
  const int64_t n_x = (int64_t)gridDim.x - n_front_blocks;
  const int64_t b = ((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * n_x + ((int64_t)blockIdx.x - n_front_blocks);
  const int wave = threadIdx.x >> 6;
  const int64_t item = b * kp + wave;
  const int64_t n_knots = (int64_t)aio.n_problems * aio.n_heads * aio.n_grid;
  return (wave < kp && item < n_knots) ? item : -1;
}

// ---- pass A: softmax statistics ----------------------------------------------------------
template <bool F32, int D, int NBM, int RG>
__global__ __launch_bounds__(256, (F32 && D == 128) ? 1 : 2) void score_stats_kernel(Geom g, SeqTab tab, AllocIO aio,
                                                          int n_alloc_blocks, int alloc_bpp, int alloc_spread,
                                                          const char* q,
                                                          const char* k, float* lpart,
                                                          int rows_padded) {
  using T = Tile<F32, D, RG>;
  constexpr int kBufRows = T::kKeys > 32 * NBM ? T::kKeys : 32 * NBM;   // K tile or one Q row group
  __shared__ u32x4 ktile[kBufRows * T::kLdsRowU4];
  __shared__ float2 wstat[4][NBM][32];

  if ((int)blockIdx.x < n_alloc_blocks) {
    // a few short extra workgroups: hull vertices of the budget allocation (no use of scores)
    if (blockIdx.y == 0 && blockIdx.z == 0 && (int)blockIdx.x / alloc_bpp < aio.n_problems)
      alloc_phase_a(aio, blockIdx.x / alloc_bpp, blockIdx.x % alloc_bpp);
    return;
  }
  int seq, ch;
  find_tile(tab, blockIdx.x - n_alloc_blocks, seq, ch);
  const int kvh = blockIdx.y, layer = blockIdx.z;
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0, P = L - g.window;
  const int hi = (seq * g.n_layers + layer) * g.n_kv_heads + kvh;
  // (the wave index is uniform over a wave: saying so keeps what derives from it in scalar registers)
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, hf = lane >> 5;
  constexpr int n_kt = T::kWaveCols;
  const int kt = wave % n_kt, rg = wave / n_kt;
  const int blk0 = rg * g.blocks_per_group;
  int nb_count = g.row_blocks - blk0;
  nb_count = nb_count < 0 ? 0 : (nb_count > g.blocks_per_group ? g.blocks_per_group : nb_count);
  const float a = g.scale_log2e;

  const char* kbase = k + ((int64_t)layer * g.sl + (int64_t)kvh * g.sh + (int64_t)tok0 * g.st) * T::kEsize;
  const int j_begin = ch * g.chunk_keys;
  const int j_end = min(L, j_begin + g.chunk_keys);
  // Spread form of the allocation's first phase: this workgroup takes up to four knots, one per
  // wave.  Their loads are issued ahead of the K tile's and consumed after the queries are on
  // their way, so the divisions run while the tile is in flight.
  const int64_t a_item = spread_item(aio, alloc_spread, n_alloc_blocks);
  AllocKnotLoad a_ld;
  // byte offsets inside one head's keys fit 32 bits (checked on the host)
  const unsigned tok_bytes = (unsigned)(g.st * T::kEsize);
  const int ld_row0 = T::kPrivate ? 32 * (int)(threadIdx.x >> 6) + (int)(threadIdx.x & 63) / T::kRowU4
                                  : (int)threadIdx.x / T::kRowU4;
  const int ld_col = threadIdx.x % T::kRowU4;
  const int ld_lds = ld_row0 * T::kLdsRowU4 + ld_col;
  const unsigned ld_stride = (unsigned)T::kLoadRowStep * tok_bytes, ld_tile = (unsigned)T::kKeys * tok_bytes;
  const unsigned ld_last = (unsigned)(L - 1) * tok_bytes + (unsigned)ld_col * 16u;
  unsigned ld_off = (unsigned)(j_begin + ld_row0) * tok_bytes + (unsigned)ld_col * 16u;
  // the window queries of the first row group are requested ahead of the first K tile (they come
  // from L2 and are parked and picked up while the tile is still on its way from HBM)
  u32x4 pre[T::kLoads];
  u32x4 qreg[NBM][T::kHalfU4];
  {
    u32x4 qtmp[QStage<F32, D, NBM>::kLoads];
    q_fetch<F32, D, NBM, QStage<F32, D, NBM>::kLoads>(qtmp, g, q, layer, kvh, seq, 0);
    k_issue<F32, D, RG, T::kLoads>(pre, kbase, ld_off, ld_stride, ld_last);
    // the allocation's knot of this wave: its loads are cold and go out last, so that nothing the
    // workgroup needs first waits behind them; they are consumed once the first tile is in LDS
    if (a_item >= 0) a_ld = alloc_knot_load(aio, a_item);
    for (int grp = 0; grp < RG; ++grp) {
      if (grp) q_fetch<F32, D, NBM, QStage<F32, D, NBM>::kLoads>(qtmp, g, q, layer, kvh, seq, grp);
      if (grp) __syncthreads();
      q_park<F32, D, NBM, QStage<F32, D, NBM>::kLoads>(qtmp, ktile);
      __syncthreads();
      if (rg == grp) q_pick<F32, D, NBM, T::kHalfU4>(qreg, ktile, lane);
    }
  }
  __syncthreads();   // the buffer now turns into the K tile

  // window row index of this lane's query in every block (for the causal range)
  int wrow[NBM];
#pragma unroll
  for (int nb = 0; nb < NBM; ++nb) wrow[nb] = (32 * (blk0 + nb) + (lane & 31)) % g.window;

  float m[NBM], z[NBM];
#pragma unroll
  for (int nb = 0; nb < NBM; ++nb) { m[nb] = -INFINITY; z[nb] = 0.f; }

  // Statistics are published per granule of keys, a function of the sequence length alone (512
  // keys, doubled until a sequence has at most 64 granules), whatever chunk the call shape gives
  // a workgroup: the merged constant of a row, and with it every score, is then bitwise the same
  // for a layer scored alone or inside a larger call.  Published value: log2 of the granule's
  // sum of exponentials, l = max * a + log2(sum).
  const int gran = granule_keys(L);
  auto publish = [&](int gidx) {
    // lane l and l^32 hold the same query rows over different keys
#pragma unroll
    for (int nb = 0; nb < NBM; ++nb) {
      const float m2 = __shfl_xor(m[nb], 32), z2 = __shfl_xor(z[nb], 32);
      merge_stats(m[nb], z[nb], m2, z2, a);
      if (lane < 32) wstat[wave][nb][lane] = make_float2(m[nb], z[nb]);
      m[nb] = -INFINITY;
      z[nb] = 0.f;
    }
    __syncthreads();
    // merge the key subtiles of every row group
    for (int r = threadIdx.x; r < rows_padded; r += 256) {
      const int blk = r >> 5, grp = blk / g.blocks_per_group, nb = blk - grp * g.blocks_per_group;
      float mm = -INFINITY, zz = 0.f;
      for (int t = 0; t < n_kt; ++t) {
        const float2 st = wstat[grp * n_kt + t][nb][r & 31];
        merge_stats(mm, zz, st.x, st.y, a);
      }
      lpart[((int64_t)hi * kMaxGranules + gidx) * rows_padded + r] = mm == -INFINITY ? -INFINITY : fmaf(mm, a, log2f(zz));
    }
    __syncthreads();   // wstat is rewritten by the next granule
  };

  // One tile.  The first one is a copy of its own (first_tag), so that the knot's registers are
  // not carried through the loop.
  auto tile = [&](int j0, auto first_tag) {
    tile_sync<T::kPrivate>();      // the previous tile has been read
    k_commit<F32, D, RG, T::kLoads>(pre, ktile, ld_lds);
    tile_sync<T::kPrivate>();
    ld_off += ld_tile;
    if (j0 + T::kKeys < j_end) k_issue<F32, D, RG, T::kLoads>(pre, kbase, ld_off, ld_stride, ld_last);
    if constexpr (decltype(first_tag)::value) {
      if (a_item >= 0) alloc_knot_finish(aio, a_item, a_ld);
    }
    const int jw = j0 + 32 * kt;   // first key of this wave's 32-key subtile
    if (jw < j_end) {              // wave-uniform
      u32x4 kreg[T::kHalfU4];
      const u32x4* src = ktile + (32 * kt + (lane & 31)) * T::kLdsRowU4 + hf * T::kHalfU4;
#pragma unroll
      for (int s = 0; s < T::kHalfU4; ++s) kreg[s] = src[s];
      // Only the last tiles of a sequence reach into the observation window (causal range) or
      // past the end; every other tile takes the branch-free path.
      auto fold = [&](auto masked_tag) {
        constexpr bool kMasked = decltype(masked_tag)::value;
#pragma unroll
        for (int nb = 0; nb < NBM; ++nb) {
          if (nb < nb_count) {
            f32x16 acc = {0};
#pragma unroll
            for (int s = 0; s < T::kHalfU4; ++s) acc = mma<F32>(kreg[s], qreg[nb][s], acc);
            if constexpr (kMasked) {
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
      };
      if (jw + 32 > P) {
        fold(std::true_type{});
      } else {
        fold(std::false_type{});
      }
    }
    const int j_next = j0 + T::kKeys;
    if (j_next >= j_end || j_next % gran == 0) publish((j_next - 1) / gran);   // uniform over the workgroup
  };
  if (j_begin < j_end) tile(j_begin, std::true_type{});
  else if (a_item >= 0) alloc_knot_finish(aio, a_item, a_ld);
  for (int j0 = j_begin + T::kKeys; j0 < j_end; j0 += T::kKeys) tile(j0, std::false_type{});
}

// ---- pass B: normalised window sums ------------------------------------------------------
template <bool F32, int D, int NBM, int RG>
__global__ __launch_bounds__(256, (F32 && D == 128) ? 1 : 2) void score_accum_kernel(Geom g, SeqTab tab, AllocIO aio,
                                                          int n_alloc_blocks, int alloc_bpp, int alloc_spread,
                                                          const char* q,
                                                          const char* k, const float* lpart,
                                                          const float* lse,
                                                          float* raw, float2* range, int max_chunks,
                                                          int rows_padded) {
  using T = Tile<F32, D, RG>;
  constexpr int kBufRows = T::kKeys > 32 * NBM ? T::kKeys : 32 * NBM;   // K tile or one Q row group
  constexpr int kBufU4 = kBufRows * T::kLdsRowU4;
  __shared__ u32x4 ktile[kBufU4];
  __shared__ __align__(16) float rowc_s[kMaxRows];
  __shared__ float2 pm[1024];
  __shared__ float colred[4][32];

  if ((int)blockIdx.x < n_alloc_blocks) {
    // Extra workgroups, dispatched first (no use of scores): the hull vertices, when there is no
    // statistics kernel to carry them.
    if (blockIdx.y == 0 && blockIdx.z == 0 && (int)blockIdx.x / alloc_bpp < aio.n_problems)
      alloc_phase_a(aio, blockIdx.x / alloc_bpp, blockIdx.x % alloc_bpp);
    return;
  }
  int seq, ch;
  find_tile(tab, blockIdx.x - n_alloc_blocks, seq, ch);
  const int kvh = blockIdx.y, layer = blockIdx.z;
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0, P = L - g.window;
  const int hi = (seq * g.n_layers + layer) * g.n_kv_heads + kvh;
  // (the wave index is uniform over a wave: saying so keeps what derives from it in scalar registers)
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, hf = lane >> 5;
  constexpr int n_kt = T::kWaveCols;
  const int kt = wave % n_kt, rg = wave / n_kt;
  const int blk0 = rg * g.blocks_per_group;
  int nb_count = g.row_blocks - blk0;
  nb_count = nb_count < 0 ? 0 : (nb_count > g.blocks_per_group ? g.blocks_per_group : nb_count);
  const float a = g.scale_log2e;

  const char* kbase = k + ((int64_t)layer * g.sl + (int64_t)kvh * g.sh + (int64_t)tok0 * g.st) * T::kEsize;
  const int j_begin = ch * g.chunk_keys;
  const int j_end = min(P, j_begin + g.chunk_keys);
  // spread form of the allocation's first phase (only when no statistics kernel carries it)
  const int64_t a_item = spread_item(aio, alloc_spread, n_alloc_blocks);
  if (a_item >= 0) alloc_knot_finish(aio, a_item, alloc_knot_load(aio, a_item));
  // byte offsets inside one head's keys fit 32 bits (checked on the host)
  const unsigned tok_bytes = (unsigned)(g.st * T::kEsize);
  const int ld_row0 = T::kPrivate ? 32 * (int)(threadIdx.x >> 6) + (int)(threadIdx.x & 63) / T::kRowU4
                                  : (int)threadIdx.x / T::kRowU4;
  const int ld_col = threadIdx.x % T::kRowU4;
  const int ld_lds = ld_row0 * T::kLdsRowU4 + ld_col;
  const unsigned ld_stride = (unsigned)T::kLoadRowStep * tok_bytes, ld_tile = (unsigned)T::kKeys * tok_bytes;
  const unsigned ld_last = (unsigned)(L - 1) * tok_bytes + (unsigned)ld_col * 16u;
  // Tiles are taken from the last to the first: pass A read them in ascending order, so its
  // last tile is the one most likely still in the L2 of this XCD when this kernel starts.
  const int n_tiles = j_end > j_begin ? (j_end - j_begin + T::kKeys - 1) / T::kKeys : 0;
  const int j_first = j_begin + (n_tiles > 0 ? n_tiles - 1 : 0) * T::kKeys;
  unsigned ld_off = (unsigned)(j_first + ld_row0) * tok_bytes + (unsigned)ld_col * 16u;
  // Requests go out in the order their answers are needed, since a wave sees its loads return
  // in order: the window queries of the first row group and the first batch of pass A's
  // statistics (both from L2), then the first K tile (from HBM, the long wait), so the queries
  // are parked and the softmax constants merged while that tile is on its way.
  u32x4 pre[T::kLoads];
  u32x4 qtmp[QStage<F32, D, NBM>::kLoads];
  q_fetch<F32, D, NBM, QStage<F32, D, NBM>::kLoads>(qtmp, g, q, layer, kvh, seq, 0);

  // Softmax constant of every window row, c_r = log2 of the row's denominator.  Either the
  // caller's log-sum-exp (row r = query head r / w of the group, window row r % w), or the merge
  // of the granules' log-sums l that pass A left, c_r = M + log2(sum exp2(l - M)), M = max l:
  // a thread takes four rows (one 16-byte load per granule) and every (256 / (rows / 4))-th
  // granule, eight loads in flight at a time; LDS joins the threads that share rows.
  if (lse) {
    k_issue<F32, D, RG, T::kLoads>(pre, kbase, ld_off, ld_stride, ld_last);
    const int64_t qh0 = (int64_t)layer * g.n_q_heads + (int64_t)kvh * g.group;
    const int64_t row_len = (int64_t)tab.n_seqs * g.window;
    for (int r = threadIdx.x; r < kMaxRows; r += 256) {
      float c = INFINITY;   // padded rows never contribute
      if (r < g.rows) c = lse[(qh0 + r / g.window) * row_len + (int64_t)seq * g.window + r % g.window] * 1.44269504088896340736f;
      rowc_s[r] = c;
    }
  } else {
    const int n_gran = (L + granule_keys(L) - 1) / granule_keys(L);
    const int tpr = rows_padded >> 2;                 // threads that cover the rows once: 8 .. 128
    const int groups = 256 / tpr;                     // 2 .. 32
    const int col = (int)threadIdx.x % tpr, grp0 = (int)threadIdx.x / tpr;
    const float* hp = lpart + (int64_t)hi * kMaxGranules * rows_padded + 4 * col;
    float pmax[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY}, psum[4] = {0.f, 0.f, 0.f, 0.f};
    f32x4 v[8];
    auto fetch8 = [&](int g0) {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int gi = g0 + u * groups;
        v[u] = gi < n_gran ? *reinterpret_cast<const f32x4*>(hp + (int64_t)gi * rows_padded)
                           : f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
      }
    };
    int g0 = grp0 < groups ? grp0 : n_gran;           // (threads beyond the last group idle)
    fetch8(g0);
    k_issue<F32, D, RG, T::kLoads>(pre, kbase, ld_off, ld_stride, ld_last);
    while (g0 < n_gran) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float bm = pmax[e];
#pragma unroll
        for (int u = 0; u < 8; ++u) bm = fmaxf(bm, v[u][e]);
        const float ref = bm == -INFINITY ? 0.f : bm;
        float bs = psum[e] * fast_exp2(pmax[e] - ref);
#pragma unroll
        for (int u = 0; u < 8; ++u) bs += fast_exp2(v[u][e] - ref);
        pmax[e] = bm;
        psum[e] = bs;
      }
      g0 += 8 * groups;
      if (g0 < n_gran) fetch8(g0);
    }
    if (grp0 < groups) {
#pragma unroll
      for (int e = 0; e < 4; ++e) pm[grp0 * rows_padded + 4 * col + e] = make_float2(pmax[e], psum[e]);
    }
    __syncthreads();
    for (int r = threadIdx.x; r < rows_padded; r += 256) {
      float bm = -INFINITY;
      for (int p2 = 0; p2 < groups; ++p2) bm = fmaxf(bm, pm[p2 * rows_padded + r].x);
      const float ref = bm == -INFINITY ? 0.f : bm;
      float bs = 0.f;
      for (int p2 = 0; p2 < groups; ++p2) {
        const float2 st = pm[p2 * rows_padded + r];
        bs = fmaf(st.y, fast_exp2(st.x - ref), bs);
      }
      // padded rows never contribute: +inf makes exp2(S*a - c) vanish
      rowc_s[r] = r < g.rows ? bm + log2f(bs) : INFINITY;
    }
    for (int r = rows_padded + threadIdx.x; r < kMaxRows; r += 256) rowc_s[r] = INFINITY;
  }

  u32x4 qreg[NBM][T::kHalfU4];
  for (int grp = 0; grp < RG; ++grp) {
    if (grp) {
      q_fetch<F32, D, NBM, QStage<F32, D, NBM>::kLoads>(qtmp, g, q, layer, kvh, seq, grp);
      __syncthreads();
    }
    q_park<F32, D, NBM, QStage<F32, D, NBM>::kLoads>(qtmp, ktile);
    __syncthreads();
    if (rg == grp) q_pick<F32, D, NBM, T::kHalfU4>(qreg, ktile, lane);
  }
  __syncthreads();   // the buffer now turns into the K tile; rowc_s is complete

  float* out = raw + ((int64_t)layer * g.n_kv_heads + kvh) * g.total_tokens + tok0;
  float vmin = INFINITY, vmax = -INFINITY;   // range of the values this lane writes

  for (int ti = n_tiles - 1; ti >= 0; --ti) {
    const int j0 = j_begin + ti * T::kKeys;
    tile_sync<T::kPrivate>();
    k_commit<F32, D, RG, T::kLoads>(pre, ktile, ld_lds);
    tile_sync<T::kPrivate>();
    ld_off -= ld_tile;
    if (ti > 0) k_issue<F32, D, RG, T::kLoads>(pre, kbase, ld_off, ld_stride, ld_last);
    const int jw = j0 + 32 * kt;
    float col = 0.f;
    if (jw < j_end) {
      u32x4 kreg[T::kHalfU4];
      const u32x4* src = ktile + (32 * kt + (lane & 31)) * T::kLdsRowU4 + hf * T::kHalfU4;
#pragma unroll
      for (int s = 0; s < T::kHalfU4; ++s) kreg[s] = src[s];
      if (nb_count == NBM && !F32) {
        // all row blocks live (wave-uniform): the softmax constants of every block are read
        // first, then the matrix products of block nb+1 are issued one at a time between the
        // exponentials of block nb (its 16 probabilities shared out over the MFMAs), so that the matrix pipe and
        // the vector ALU of this wave run side by side
        f32x16 acc = {0};
#pragma unroll
        for (int s = 0; s < T::kHalfU4; ++s) acc = mma<F32>(qreg[0][s], kreg[s], acc);
#pragma unroll
        for (int nb = 0; nb < NBM; ++nb) {
          f32x16 nxt = {0};
          f32x4 cst[1][4];
#pragma unroll
          for (int v4 = 0; v4 < 4; ++v4)
            cst[0][v4] = *reinterpret_cast<const f32x4*>(rowc_s + 32 * (blk0 + nb) + 4 * hf + 8 * v4);
#pragma unroll
          for (int s = 0; s < T::kHalfU4; ++s) {
            if (nb + 1 < NBM) nxt = mma<F32>(qreg[nb + 1][s], kreg[s], nxt);
            // this step's share of the finished block's 16 elements
            constexpr int kEl = 16 / T::kHalfU4;
#pragma unroll
            for (int e = s * kEl; e < (s + 1) * kEl; ++e) col += fast_exp2(fmaf(acc[e], a, -cst[0][e >> 2][e & 3]));
            if (nb + 1 < NBM) {
              __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);          // one MFMA
              __builtin_amdgcn_sched_group_barrier(0x402, 3 * kEl, 0);    // kEl x (fma, exp2, add)
            }
          }
          acc = nxt;
        }
      } else {
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
      }
      col += __shfl_xor(col, 32);
    }
    if (RG > 1) {
      // fixed-order sum over the row groups keeps the result deterministic
      if (lane < 32) colred[wave][lane] = col;
      __syncthreads();
      if (rg == 0) {
#pragma unroll
        for (int t = 1; t < RG; ++t) col += colred[t * n_kt + kt][lane & 31];
      }
    }
    // (the lane index is taken afresh here: kept in a register across the products above it
    // would be the one value too many and go through scratch memory)
    int ln;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(ln));
    if (rg == 0 && ln < 32 && jw + ln < j_end) {
      const float val = col * g.inv_group;
      out[jw + ln] = val;
      vmin = fminf(vmin, val);
      vmax = fmaxf(vmax, val);
    }
  }
  // Value range of the chunk, one entry per wave (neutral where a wave wrote nothing): the
  // selection scales its first radix digit to the range of the head's metric.
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) {
    vmin = fminf(vmin, __shfl_xor(vmin, o));
    vmax = fmaxf(vmax, __shfl_xor(vmax, o));
  }
  int ln0;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(ln0));
  if (ln0 == 0) range[((int64_t)hi * max_chunks + ch) * 4 + wave] = make_float2(vmin, vmax);
}

// ---- pooling + forced positions (stand-alone scores) -------------------------------------
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

// ---- launchers ---------------------------------------------------------------------------
template <bool F32, int D, int NBM, int RG>
static int launch_raw_t(const HostCfg& hc, const WsLayout& lay, const void* q, const void* k,
                        const float* lse, const AllocIO* aio, char* ws, hipStream_t st) {
  const Geom& g = hc.g;
  float* lpart = reinterpret_cast<float*>(ws + lay.partial);
  float* raw = reinterpret_cast<float*>(ws + lay.raw);
  float2* range = reinterpret_cast<float2*>(ws + lay.range);
  const SeqTab tabA = tiles_for(hc.seq, g.chunk_keys, 0);
  const SeqTab tabB = tiles_for(hc.seq, g.chunk_keys, g.window);
  AllocIO io;
  memset(&io, 0, sizeof(io));
  // The allocation never looks at scores, so its first phase (hull vertices) rides in the score
  // kernels: spread over the prologues of the statistics kernel's workgroups, one knot per wave,
  // when there are enough of them; else a few extra workgroups at the front of its grid.  Without
  // a statistics kernel (log-sum-exp supplied) the accumulation kernel carries it the same way.
  // Extra workgroups are padded to a multiple of 8 so that a chunk lands on the same XCD (and its
  // L2) in both passes.
  const int64_t wgsA = (int64_t)tabA.tile0[tabA.n_seqs] * g.n_kv_heads * g.n_layers;
  const int64_t wgsB = (int64_t)tabB.tile0[tabB.n_seqs] * g.n_kv_heads * g.n_layers;
  int frontA = 0, bppA = 1, spreadA = 0, frontB = 0, bppB = 1, spreadB = 0;
  if (aio) {
    io = *aio;
    const int64_t n_knots = (int64_t)aio->n_problems * aio->n_heads * aio->n_grid;
    const int bpp = alloc_blocks_a(aio->n_heads, aio->n_grid);
    if (!lse) {
      spreadA = alloc_spread_knots(n_knots, wgsA);
      if (!spreadA) { bppA = bpp; frontA = (aio->n_problems * bpp + 7) / 8 * 8; }
    } else {
      spreadB = alloc_spread_knots(n_knots, wgsB);
      if (!spreadB) { bppB = bpp; frontB = (aio->n_problems * bpp + 7) / 8 * 8; }
    }
  }
  dim3 gridA(tabA.tile0[tabA.n_seqs] + frontA, g.n_kv_heads, g.n_layers);
  dim3 gridB(tabB.tile0[tabB.n_seqs] + frontB, g.n_kv_heads, g.n_layers);
  if (!lse)
    launch_staged(kStStats, score_stats_kernel<F32, D, NBM, RG>, gridA, dim3(256), st, g, tabA, io, frontA, bppA,
                  spreadA, (const char*)q, (const char*)k, lpart, lay.rows_padded);
  launch_staged(kStAccum, score_accum_kernel<F32, D, NBM, RG>, gridB, dim3(256), st, g, tabB, io,
                frontB, bppB, spreadB, (const char*)q, (const char*)k, (const float*)lpart, lse, raw,
                range, lay.max_chunks, lay.rows_padded);
  return check_launch();
}

template <bool F32, int D, int NBM>
static int launch_raw_rg(const HostCfg& hc, const WsLayout& lay, const void* q, const void* k,
                         const float* lse, const AllocIO* aio, char* ws, hipStream_t st) {
  switch (hc.g.row_groups) {
    case 1: return launch_raw_t<F32, D, NBM, 1>(hc, lay, q, k, lse, aio, ws, st);
    case 2: return launch_raw_t<F32, D, NBM, 2>(hc, lay, q, k, lse, aio, ws, st);
    case 4: return launch_raw_t<F32, D, NBM, 4>(hc, lay, q, k, lse, aio, ws, st);
  }
  return LUKV_EINVAL;
}

int launch_score_raw(const HostCfg& hc, const WsLayout& lay, const void* q, const void* k,
                     const float* lse, const AllocIO* aio, char* ws, hipStream_t st) {
  const Geom& g = hc.g;
  if (!g.f32 && g.head_dim == 128) return launch_raw_rg<false, 128, 4>(hc, lay, q, k, lse, aio, ws, st);
  if (!g.f32 && g.head_dim == 64) return launch_raw_rg<false, 64, 4>(hc, lay, q, k, lse, aio, ws, st);
  if (g.f32 && g.head_dim == 64) return launch_raw_rg<true, 64, 4>(hc, lay, q, k, lse, aio, ws, st);
  if (g.f32 && g.head_dim == 128) return launch_raw_rg<true, 128, 2>(hc, lay, q, k, lse, aio, ws, st);
  return LUKV_EDTYPE;
}

int launch_pool(const HostCfg& hc, const WsLayout& lay, float* pooled_out, char* ws, hipStream_t st) {
  const Geom& g = hc.g;
  const SeqTab tabP = tiles_for(hc.seq, 256, 0);
  dim3 gridP(tabP.tile0[tabP.n_seqs], g.n_kv_heads * g.n_layers, 1);
  launch_staged(kStPool, pool_kernel, gridP, dim3(256), st, g, tabP,
                reinterpret_cast<const float*>(ws + lay.raw), pooled_out);
  return check_launch();
}

}  // namespace lukv
