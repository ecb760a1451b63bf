// Offline profiling, first step (Sec. 4.1, Eq. 6): the utility curve of a head from per-token
// importance and the heuristic metric's ranking.  One workgroup per curve: the tokens are sorted
// by (score descending, index ascending) with a bitonic network in LDS, the importance is summed
// along that ranking in fp64, and the running sum is sampled at the caller's knots.
#include "lukv_internal.hpp"

namespace lukv {

constexpr int kCurveMaxT = 4096;   // tokens per profiled context (one LDS-resident sort)

__device__ __forceinline__ unsigned curve_key(float f) {
  unsigned u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;  // -0 and +0 tie
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(1024) void profile_curves_kernel(const float* importance, const float* scores,
                                                              const int32_t* knots, int T, int n_grid,
                                                              float* curves) {
  __shared__ unsigned long long keys[kCurveMaxT + 8];   // the ranking, then the running sums
  __shared__ double wave_tot[16];
  const int c = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const float* imp = importance + (int64_t)c * T;
  const float* sc = scores + (int64_t)c * T;
  // larger composite = earlier in the ranking: higher score, then lower index; padding sorts last
  for (int i = t; i < kCurveMaxT; i += 1024)
    keys[i] = i < T ? ((unsigned long long)curve_key(sc[i]) << 32) | (0xFFFFFFFFu - (unsigned)i) : 0ull;
  __syncthreads();
  for (int k = 2; k <= kCurveMaxT; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
#pragma unroll
      for (int u = 0; u < kCurveMaxT / 2048; ++u) {
        const int q = t + 1024 * u;
        const int i = 2 * q - (q & (j - 1)), l = i + j;
        const unsigned long long a = keys[i], b = keys[l];
        const bool down = (i & k) == 0;              // this run is sorted descending
        if (down ? a < b : a > b) { keys[i] = b; keys[l] = a; }
      }
      __syncthreads();
    }
  }
  // importance along the ranking: four consecutive ranks per thread, fp64
  double v[4], run = 0.0;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int r = 4 * t + e;
    const unsigned idx = 0xFFFFFFFFu - (unsigned)keys[r];
    run += r < T ? (double)imp[idx] : 0.0;
    v[e] = run;
  }
  double incl = run;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const long long bits = __double_as_longlong(incl);
    const int lo = __shfl_up((int)(bits & 0xFFFFFFFFll), o), hi = __shfl_up((int)(bits >> 32), o);
    const double up = __longlong_as_double(((long long)hi << 32) | (unsigned)lo);
    if (lane >= o) incl += up;
  }
  __syncthreads();                                   // every rank has been read
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  double before = incl - run;
  for (int w = 0; w < wave; ++w) before += wave_tot[w];
  double* pre = reinterpret_cast<double*>(keys);     // pre[r] = mass of the first r tokens
  if (t == 0) pre[0] = 0.0;
#pragma unroll
  for (int e = 0; e < 4; ++e) pre[4 * t + e + 1] = before + v[e];
  __syncthreads();
  for (int g = t; g < n_grid; g += 1024) {
    int n = knots[(int64_t)c * n_grid + g];
    n = n < 0 ? 0 : (n > T ? T : n);
    curves[(int64_t)c * n_grid + g] = (float)pre[n];
  }
}

int launch_profile_curves(int32_t n_curves, int32_t T, int32_t n_grid, const float* importance,
                          const float* scores, const int32_t* knots, float* curves, hipStream_t st) {
  if (T > kCurveMaxT) return LUKV_EINVAL;
  hipLaunchKernelGGL(profile_curves_kernel, dim3(n_curves), dim3(1024), 0, st, importance, scores, knots, T,
                     n_grid, curves);
  return check_launch();
}

}  // namespace lukv
