// Instrumentation of liblukv (include/lukv_bench.h): per-stage start / stop events for callers
// that time the path, and two plain streaming kernels of known size that measure what this GPU
// sustains beside the nominal HBM peak.  Nothing of the method lives here.
#include "lukv_bench.h"
#include "lukv_internal.hpp"

namespace lukv {

static void* const* g_stage_events = nullptr;
static int g_n_stage_events = 0;

void stage_events(int stage, hipEvent_t* start, hipEvent_t* stop) {
  *start = *stop = nullptr;
  if (!g_stage_events) return;
  if (2 * stage < g_n_stage_events) *start = static_cast<hipEvent_t>(g_stage_events[2 * stage]);
  if (2 * stage + 1 < g_n_stage_events) *stop = static_cast<hipEvent_t>(g_stage_events[2 * stage + 1]);
}

// every 16-byte word once, grid-strided, eight loads in flight per thread; one word per wave
// goes to the sink so that the loads cannot be dropped
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* src, int64_t n16, unsigned* sink) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  unsigned acc = 0;
  for (; i + 7 * stride < n16; i += 8 * stride) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n16; i += stride) acc += src[i].x;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
  if ((threadIdx.x & 63) == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = acc;
}

__global__ __launch_bounds__(256) void copy_kernel(const u32x4* src, u32x4* dst, int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a;
    dst[i + stride] = b;
    dst[i + 2 * stride] = c;
    dst[i + 3 * stride] = d;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace lukv

using namespace lukv;

extern "C" {

int lukv_set_stage_events(void* const* events, int32_t n_events) {
  if (n_events < 0 || (n_events > 0 && !events)) return LUKV_EINVAL;
  g_stage_events = n_events ? events : nullptr;
  g_n_stage_events = n_events;
  return LUKV_OK;
}

const char* lukv_stage_name(int32_t stage) {
  static const char* const names[kNumStages] = {
      "allocate", "score_stats", "score_accum", "pool", "sel_hist", "sel_tail", "sel_emit", "sel_head", "sel_gather"};
  return stage >= 0 && stage < kNumStages ? names[stage] : "";
}

static bool bench_args_ok(const void* a, const void* b, int64_t bytes, int32_t blocks) {
  return a && b && bytes > 0 && bytes % 16 == 0 && blocks >= 1 && blocks <= 65536 &&
         (reinterpret_cast<uintptr_t>(a) & 15u) == 0 && (reinterpret_cast<uintptr_t>(b) & 3u) == 0;
}

int lukv_bench_stream_read(const void* src, int64_t bytes, void* sink, int32_t blocks, void* stream) {
  if (!bench_args_ok(src, sink, bytes, blocks)) return LUKV_EINVAL;
  hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(src), bytes / 16, static_cast<unsigned*>(sink));
  return check_launch();
}

int lukv_bench_copy(const void* src, void* dst, int64_t bytes, int32_t blocks, void* stream) {
  if (!bench_args_ok(src, dst, bytes, blocks) || (reinterpret_cast<uintptr_t>(dst) & 15u)) return LUKV_EINVAL;
  hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), bytes / 16);
  return check_launch();
}

}  // extern "C"
