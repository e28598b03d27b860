// Expert SwiGLU FFN (paper section 2, Eq. 3) and the weighted sum of Eq. 2 for
// expert blocks kept in the plain row-major layout W_g | W_u | W_d, fp32 or
// bf16.  This is the layout-agnostic path (one wavefront per output row, DPP
// reduction over the contraction); the bf16 production path is ffn_tiled.hip.
#include "device_utils.hpp"
#include "moe_internal.hpp"

namespace moe {

namespace {

constexpr int kRowsPerBlock = 4;

__device__ __forceinline__ const char* group_weights(const FfnArgs& a, int id) {
  return id < a.P ? a.buffers + (size_t)id * a.expert_bytes
                  : a.shared + (size_t)(id - a.P) * a.expert_bytes;
}

// h[pos][j] = silu(W_g[j,:].x) * (W_u[j,:].x)
template <typename T>
__global__ void __launch_bounds__(64 * kRowsPerBlock) gate_up_rowmajor(FfnArgs a) {
  const int g = blockIdx.y;
  const int ng = *a.t.n_groups;
  const GroupDesc gd = a.t.grp[g];
  if (g >= ng || (a.pass != 2 && gd.miss != a.pass)) return;
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (j >= a.f) return;
  const T* w = reinterpret_cast<const T*>(group_weights(a, gd.buf));
  const T* wg = w + (size_t)j * a.d;
  const T* wu = w + (size_t)a.f * a.d + (size_t)j * a.d;
  const int begin = gd.begin, cnt = gd.count;
  float* h = reinterpret_cast<float*>(a.h);
  for (int tkn = 0; tkn < cnt; ++tkn) {
    const int p = a.t.sorted_pair[begin + tkn];
    const T* xr = reinterpret_cast<const T*>(a.x) + (size_t)(p / a.KS) * a.d;
    float sg = 0.f, su = 0.f;
    for (int i = lane; i < a.d; i += kWave) {
      const float xv = Elem<T>::load(xr + i);
      sg = fmaf(Elem<T>::load(wg + i), xv, sg);
      su = fmaf(Elem<T>::load(wu + i), xv, su);
    }
    sg = wave_sum(sg);
    su = wave_sum(su);
    if (lane == 0) h[(size_t)(begin + tkn) * a.f + j] = silu(sg) * su;
  }
}

// o[pos][i] = W_d[i,:].h[pos,:]
template <typename T>
__global__ void __launch_bounds__(64 * kRowsPerBlock) down_rowmajor(FfnArgs a) {
  const int g = blockIdx.y;
  const int ng = *a.t.n_groups;
  const GroupDesc gd = a.t.grp[g];
  if (g >= ng || (a.pass != 2 && gd.miss != a.pass)) return;
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (i >= a.d) return;
  const T* wd = reinterpret_cast<const T*>(group_weights(a, gd.buf)) + (size_t)2 * a.f * a.d + (size_t)i * a.f;
  const int begin = gd.begin, cnt = gd.count;
  const float* h = reinterpret_cast<const float*>(a.h);
  for (int tkn = 0; tkn < cnt; ++tkn) {
    const float* hr = h + (size_t)(begin + tkn) * a.f;
    float s = 0.f;
    for (int j = lane; j < a.f; j += kWave) s = fmaf(Elem<T>::load(wd + j), hr[j], s);
    s = wave_sum(s);
    if (lane == 0) a.o[(size_t)(begin + tkn) * a.d + i] = s;
  }
}

// y[b][i] = sum_j wpair[b][j] * o[pos_of[b][j]][i], j over the K selected then the shared experts.
// A thread owns four consecutive columns (16-byte loads); the rows of a batch of pairs are all requested before
// the first is used; the pairs are added in index order, so the result does not depend on the batch size.
typedef float f32x4_c __attribute__((ext_vector_type(4)));
constexpr int kCombinePairs = 8;

template <typename T>
__global__ void __launch_bounds__(256)
combine_kernel(const float* __restrict__ o, const float* __restrict__ wpair, const int32_t* __restrict__ pos_of,
               int KS, int d, T* __restrict__ y) {
  const int b = blockIdx.x;
  const int i = (blockIdx.y * blockDim.x + threadIdx.x) * 4;      // host guarantees d % 4 == 0
  if (i >= d) return;
  const float* wrow = wpair + (size_t)b * KS;
  const int32_t* prow = pos_of + (size_t)b * KS;
  f32x4_c acc = {0.f, 0.f, 0.f, 0.f};
  for (int j0 = 0; j0 < KS; j0 += kCombinePairs) {
    f32x4_c v[kCombinePairs];
    float w[kCombinePairs];
#pragma unroll
    for (int u = 0; u < kCombinePairs; ++u) {
      const int j = j0 + u < KS ? j0 + u : KS - 1;          // clamped: in bounds, weight zeroed below
      w[u] = j0 + u < KS ? wrow[j] : 0.f;
      v[u] = *reinterpret_cast<const f32x4_c*>(o + (size_t)prow[j] * d + i);
    }
#pragma unroll
    for (int u = 0; u < kCombinePairs; ++u) {
      if (j0 + u < KS) {      // uniform
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] = fmaf(w[u], v[u][c], acc[c]);
      }
    }
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) Elem<T>::store(y + (size_t)b * d + i + c, acc[c]);
}

}  // namespace

hipError_t launch_ffn_rowmajor(hipStream_t s, int dtype, const FfnArgs& a, KernelEvents e1, KernelEvents e2) {
  if (a.g_max <= 0) return hipSuccess;
  dim3 block(64 * kRowsPerBlock);
  dim3 g1((a.f + kRowsPerBlock - 1) / kRowsPerBlock, a.g_max);
  dim3 g2((a.d + kRowsPerBlock - 1) / kRowsPerBlock, a.g_max);
  if (dtype == MOE_DTYPE_FP32) {
    launch_timed(gate_up_rowmajor<float>, g1, block, 0, s, e1, a);
    launch_timed(down_rowmajor<float>, g2, block, 0, s, e2, a);
  } else {
    launch_timed(gate_up_rowmajor<uint16_t>, g1, block, 0, s, e1, a);
    launch_timed(down_rowmajor<uint16_t>, g2, block, 0, s, e2, a);
  }
  return hipGetLastError();
}

hipError_t launch_combine(hipStream_t s, int dtype, const float* o, const float* wpair, const int32_t* pos_of,
                          int B, int KS, int d, void* y) {
  dim3 grid(B, (d / 4 + 255) / 256), block(256);
  if (dtype == MOE_DTYPE_FP32)
    hipLaunchKernelGGL(combine_kernel<float>, grid, block, 0, s, o, wpair, pos_of, KS, d, (float*)y);
  else
    hipLaunchKernelGGL(combine_kernel<uint16_t>, grid, block, 0, s, o, wpair, pos_of, KS, d, (uint16_t*)y);
  return hipGetLastError();
}

}  // namespace moe
