// Stand-alone kernel and launch helpers for step 2 (the device code is in alloc_device.hpp;
// the fused path runs the same two phases as extra workgroups of the score kernels).
#include "alloc_device.hpp"

namespace lukv {

__global__ __launch_bounds__(256) void allocate_vertices_kernel(AllocIO io, int blocks_per_problem) {
  alloc_phase_a(io, blockIdx.x / blocks_per_problem, blockIdx.x % blocks_per_problem);
}

__global__ __launch_bounds__(1024) void allocate_budgets_kernel(AllocIO io) {
  __shared__ __align__(16) char lds[kAllocLdsBytes];
  alloc_phase_b(io, blockIdx.x, lds, (int)sizeof(lds));
}

// offsets = exclusive prefix sum of all budgets (stand-alone call; one workgroup)
__global__ __launch_bounds__(256) void offsets_kernel(const int32_t* budgets, int64_t* offsets, int64_t n_all) {
  __shared__ long long sm[4];
  long long run = 0;
  for (int64_t i0 = 0; i0 < n_all; i0 += 256) {
    const int64_t i = i0 + threadIdx.x;
    const long long b = i < n_all ? (long long)budgets[i] : 0;
    long long tot;
    const long long ex = run + block_scan_i64(b, sm, &tot);
    if (i < n_all) offsets[i] = ex;
    run += tot;
  }
  if (threadIdx.x == 0) offsets[n_all] = run;
}

// Eq. 11, one grid ratio: phi_row[h] = mean over the calibration queries of the local ratio
// 1 - b / L (fp64 sum over the queries in order, one division by M, rounded to float).
__global__ __launch_bounds__(256) void profile_accumulate_kernel(const int32_t* budgets, int n_queries,
                                                                 int n_heads, int L, float* phi_row) {
  const int h = blockIdx.x * 256 + threadIdx.x;
  if (h >= n_heads) return;
  double acc = 0.0;
  for (int m = 0; m < n_queries; ++m) acc = acc + (1.0 - (double)budgets[(int64_t)m * n_heads + h] / (double)L);
  phi_row[h] = (float)(acc / (double)n_queries);
}

// "Online Execution" steps 1-2: r = lo + t * (hi - lo) between two rows of the profile (the host
// picked the rows and t), b = floor((1 - r) * L) kept inside [b_min, b_max].
__global__ __launch_bounds__(256) void profile_lookup_kernel(const float* row_lo, const float* row_hi, double t,
                                                             int n_heads, int L, const int32_t* b_min,
                                                             const int32_t* b_max, int32_t* budgets) {
  const int h = blockIdx.x * 256 + threadIdx.x;
  if (h >= n_heads) return;
  const double lo = (double)row_lo[h];
  double r = lo;
  if (row_hi != row_lo) r = lo + t * ((double)row_hi[h] - lo);
  long long b = (long long)floor((1.0 - r) * (double)L);
  const long long mn = b_min[h], mx = b_max[h];
  b = b < mn ? mn : b;
  b = b > mx ? mx : b;
  budgets[h] = (int32_t)b;
}

int launch_profile_build(const AllocIO& io0, int32_t L, int32_t n_rho, const double* rho, float* phi,
                         hipStream_t st) {
  AllocIO io = io0;
  const int bpp = alloc_blocks_a(io.n_heads, io.n_grid);
  // the hull vertices depend on the curves only: once for all ratios
  hipLaunchKernelGGL(allocate_vertices_kernel, dim3(io.n_problems * bpp), dim3(256), 0, st, io, bpp);
  for (int r = 0; r < n_rho; ++r) {
    double B = floor((1.0 - rho[r]) * (double)L * (double)io.n_heads);
    if (!(B > 0.0)) B = 0.0;
    for (int m = 0; m < io.n_problems; ++m) io.B[m] = (int64_t)B;
    hipLaunchKernelGGL(allocate_budgets_kernel, dim3(io.n_problems), dim3(1024), 0, st, io);
    hipLaunchKernelGGL(profile_accumulate_kernel, dim3((io.n_heads + 255) / 256), dim3(256), 0, st,
                       (const int32_t*)io.budgets, io.n_problems, io.n_heads, L,
                       phi + (int64_t)r * io.n_heads);
  }
  return check_launch();
}

int launch_profile_lookup(const float* row_lo, const float* row_hi, double t, int32_t n_heads, int32_t L,
                          const int32_t* b_min, const int32_t* b_max, int32_t* budgets, int64_t* offsets,
                          hipStream_t st) {
  hipLaunchKernelGGL(profile_lookup_kernel, dim3((n_heads + 255) / 256), dim3(256), 0, st, row_lo, row_hi, t,
                     n_heads, L, b_min, b_max, budgets);
  hipLaunchKernelGGL(offsets_kernel, dim3(1), dim3(256), 0, st, (const int32_t*)budgets, offsets,
                     (int64_t)n_heads);
  return check_launch();
}

AllocIO make_alloc_io(int32_t n_problems, int32_t n_heads, int32_t n_grid, const float* curves,
                      const int32_t* knots, const int32_t* b_min, const int32_t* b_max,
                      const int64_t* B_total, int32_t* budgets, int64_t* offsets, int32_t* status,
                      const WsLayout& lay, char* ws) {
  AllocIO io;
  io.n_problems = n_problems;
  io.n_heads = n_heads;
  io.n_grid = n_grid;
  io.curves = curves;
  io.knots = knots;
  io.b_min = b_min;
  io.b_max = b_max;
  io.budgets = budgets;
  io.offsets = offsets;
  io.status = status;
  io.seg_key = reinterpret_cast<unsigned long long*>(ws + lay.seg_key);
  io.seg_w = reinterpret_cast<unsigned*>(ws + lay.seg_w);
  io.vertex = reinterpret_cast<int32_t*>(ws + lay.alloc_vertex);
  for (int i = 0; i < LUKV_MAX_SEQS; ++i) io.B[i] = (B_total && i < n_problems) ? B_total[i] : 0;
  return io;
}

void launch_offsets(const int32_t* budgets, int64_t* offsets, int64_t n_all, hipStream_t st) {
  hipLaunchKernelGGL(offsets_kernel, dim3(1), dim3(256), 0, st, budgets, offsets, n_all);
}

void launch_allocate_budgets(const AllocIO& io, hipStream_t st) {
  launch_staged(kStAllocate, allocate_budgets_kernel, dim3(io.n_problems), dim3(1024), st, io);
}

int launch_allocate(const AllocIO& io, hipStream_t st) {
  const int bpp = alloc_blocks_a(io.n_heads, io.n_grid);
  hipLaunchKernelGGL(allocate_vertices_kernel, dim3(io.n_problems * bpp), dim3(256), 0, st, io, bpp);
  launch_staged(kStAllocate, allocate_budgets_kernel, dim3(io.n_problems), dim3(1024), st, io);
  hipLaunchKernelGGL(offsets_kernel, dim3(1), dim3(256), 0, st, (const int32_t*)io.budgets, io.offsets,
                     (int64_t)io.n_problems * io.n_heads);
  return check_launch();
}

}  // namespace lukv
