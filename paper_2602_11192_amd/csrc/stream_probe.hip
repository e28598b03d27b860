// Calibration kernels: a plain streaming read and a plain copy of a buffer of
// known size.  They give (a) the HBM bandwidth this GPU actually sustains for
// the access pattern of the expert kernels (wave-wide 16-byte loads, one KiB
// per instruction) and (b) the reference dispatch for scaling the memory
// counters of a profiler run.  Not part of the decode path.
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe_cache.h"

namespace {

// every wave reads `per_wave` consecutive KiB blocks, all loads issued before the first use
template <int UNROLL>
__global__ void __launch_bounds__(512) stream_read_kernel(const uint4* __restrict__ src, size_t n_vec, uint4* sink) {
  const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  const size_t base = wave * (size_t)UNROLL * 64 + lane;
  uint4 v[UNROLL];
#pragma unroll
  for (int i = 0; i < UNROLL; ++i) {
    const size_t j = base + (size_t)i * 64;
    v[i] = j < n_vec ? src[j] : uint4{0, 0, 0, 0};
  }
  uint32_t acc = 0;
#pragma unroll
  for (int i = 0; i < UNROLL; ++i) acc ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
  if (acc == 0x9e3779b9u && sink) sink[0] = uint4{acc, 0, 0, 0};   // keeps the loads alive; practically never taken
}

__global__ void __launch_bounds__(256) copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n_vec) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_vec) dst[i] = src[i];
}

}  // namespace

extern "C" int moe_probe_stream(void* src_dev, void* dst_dev, uint64_t bytes, int32_t mode, int32_t iters,
                                void* hip_stream, double* avg_ms) {
  if (!src_dev || !avg_ms || bytes < 16 || iters < 1 || (mode != 0 && mode != 1) || (mode == 1 && !dst_dev))
    return MOE_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const size_t n_vec = bytes / 16;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return MOE_ERR_HIP;
  double total = 0.0;
  int rc = MOE_OK;
  for (int it = 0; it < iters + 1 && rc == MOE_OK; ++it) {      // first launch is a warm-up
    if (mode == 0) {
      constexpr int U = 16;
      const size_t waves = (n_vec + (size_t)U * 64 - 1) / ((size_t)U * 64);
      const size_t blocks = (waves + 7) / 8;
      hipExtLaunchKernelGGL(stream_read_kernel<U>, dim3((unsigned)blocks), dim3(512), 0, s, e0, e1, 0,
                            static_cast<const uint4*>(src_dev), n_vec, static_cast<uint4*>(dst_dev));
    } else {
      hipExtLaunchKernelGGL(copy_kernel, dim3((unsigned)((n_vec + 255) / 256)), dim3(256), 0, s, e0, e1, 0,
                            static_cast<const uint4*>(src_dev), static_cast<uint4*>(dst_dev), n_vec);
    }
    float ms = 0.f;
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = MOE_ERR_HIP;
    if (it > 0) total += ms;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  *avg_ms = total / iters;
  return rc;
}
