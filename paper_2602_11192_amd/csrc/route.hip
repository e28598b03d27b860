// Router GEMV + softmax + Top-K gating (paper section 2, Eq. 1 and the gate
// weights of Eq. 2).
//
// One workgroup per token.  Its waves split the E router rows: each wave forms
// whole dot products W_r[e,:].x with 16-byte loads and a DPP reduction, so a
// single decode token still pulls the router matrix with many loads in flight.
// Wave 0 then owns the token: each lane holds up to four logits, ranks them
// against all others (ties to the lower id), and computes the softmax with
// wave reductions.  Selection is made on the logits, which is the same set as
// Top-K of the probabilities.  Outputs are in ascending expert id.
#include "device_utils.hpp"
#include "moe_internal.hpp"

namespace moe {

constexpr int kMaxEPL = 16;  // experts per lane in the gating stage: E <= 1024

template <typename T> struct Vec;
template <> struct Vec<float> {
  static constexpr int N = 4;
  using type = float4;
  static __device__ __forceinline__ float dot(const float4& a, const float4& b, float acc) {
    acc = fmaf(a.x, b.x, acc); acc = fmaf(a.y, b.y, acc);
    acc = fmaf(a.z, b.z, acc); acc = fmaf(a.w, b.w, acc);
    return acc;
  }
};
template <> struct Vec<uint16_t> {
  static constexpr int N = 8;
  using type = uint4;
  static __device__ __forceinline__ float dot(const uint4& a, const uint4& b, float acc) {
    const uint32_t av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc = fmaf(__builtin_bit_cast(float, av[i] << 16), __builtin_bit_cast(float, bv[i] << 16), acc);
      acc = fmaf(__builtin_bit_cast(float, av[i] & 0xffff0000u),
                 __builtin_bit_cast(float, bv[i] & 0xffff0000u), acc);
    }
    return acc;
  }
};

template <typename T>
__global__ void __launch_bounds__(1024)
route_kernel(const T* __restrict__ x, const T* __restrict__ wr, const float* __restrict__ bias,
             int E, int K, int KS, int d, int norm_topk, int32_t* __restrict__ idx,
             float* __restrict__ wpair, int32_t* __restrict__ user_idx, float* __restrict__ user_w) {
  extern __shared__ float s_logit[];  // [E]
  const int b = blockIdx.x;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n_waves = blockDim.x >> 6;
  using V = Vec<T>;
  const int n_vec = d / V::N;  // host guarantees d % V::N == 0
  const typename V::type* xv = reinterpret_cast<const typename V::type*>(x + (size_t)b * d);

  for (int e = wave; e < E; e += n_waves) {
    const typename V::type* wv = reinterpret_cast<const typename V::type*>(wr + (size_t)e * d);
    float acc = 0.f;
    for (int c = lane; c < n_vec; c += kWave) acc = V::dot(wv[c], xv[c], acc);
    acc = wave_sum(acc);
    if (lane == 0) s_logit[e] = acc + (bias ? bias[(size_t)b * E + e] : 0.f);
  }
  __syncthreads();
  if (wave != 0) return;

  // ---- gating: lane l owns experts l, l+64, ... ----
  float z[kMaxEPL];
  int rank[kMaxEPL];
  const int epl = (E + kWave - 1) / kWave;
  float zmax = -INFINITY;
#pragma unroll
  for (int i = 0; i < kMaxEPL; ++i) {
    const int e = lane + i * kWave;
    z[i] = (i < epl && e < E) ? s_logit[e] : -INFINITY;
    rank[i] = 0;
    zmax = fmaxf(zmax, z[i]);
  }
  zmax = wave_max(zmax);
  for (int j = 0; j < E; ++j) {
    const float zj = s_logit[j];  // same address in every lane: LDS broadcast
#pragma unroll
    for (int i = 0; i < kMaxEPL; ++i) {
      if (i < epl) {
        const int e = lane + i * kWave;
        rank[i] += (zj > z[i] || (zj == z[i] && j < e)) ? 1 : 0;
      }
    }
  }
  float p[kMaxEPL];
  float psum = 0.f;
#pragma unroll
  for (int i = 0; i < kMaxEPL; ++i) {
    const int e = lane + i * kWave;
    p[i] = (i < epl && e < E) ? expf(z[i] - zmax) : 0.f;
    psum += p[i];
  }
  psum = wave_sum(psum);
  float selsum = 0.f;
#pragma unroll
  for (int i = 0; i < kMaxEPL; ++i) {
    const int e = lane + i * kWave;
    const bool sel = (i < epl && e < E && rank[i] < K);
    p[i] = p[i] / psum;
    selsum += sel ? p[i] : 0.f;
  }
  selsum = wave_sum(selsum);
  int base = 0;
#pragma unroll
  for (int i = 0; i < kMaxEPL; ++i) {
    if (i < epl) {  // uniform
      const int e = lane + i * kWave;
      const bool sel = (e < E && rank[i] < K);
      const uint64_t m = __ballot(sel);
      if (sel) {
        const int pos = base + __popcll(m & ((1ull << lane) - 1ull));
        const float w = norm_topk ? p[i] / selsum : p[i];
        idx[(size_t)b * K + pos] = e;
        wpair[(size_t)b * KS + pos] = w;
        if (user_idx) user_idx[(size_t)b * K + pos] = e;
        if (user_w) user_w[(size_t)b * K + pos] = w;
      }
      base += __popcll(m);
    }
  }
  if (lane < KS - K) wpair[(size_t)b * KS + K + lane] = 1.0f;  // shared experts: weight 1
}

hipError_t launch_route(hipStream_t s, int dtype, const void* x, const void* router_w, const float* bias,
                        int B, int E, int K, int KS, int d, int norm_topk, int32_t* idx, float* wpair,
                        int32_t* user_idx, float* user_w) {
  // Few tokens: 16 waves per token so the router rows stream with many loads in
  // flight.  Many tokens: fewer waves each, the grid supplies the parallelism.
  int waves = B <= 64 ? 16 : (B <= 512 ? 8 : 4);
  if (waves > E) waves = E < 1 ? 1 : E;
  dim3 grid(B), block(64 * waves);
  const size_t lds = (size_t)E * sizeof(float);
  if (dtype == MOE_DTYPE_FP32)
    hipLaunchKernelGGL(route_kernel<float>, grid, block, lds, s, (const float*)x, (const float*)router_w,
                       bias, E, K, KS, d, norm_topk, idx, wpair, user_idx, user_w);
  else
    hipLaunchKernelGGL(route_kernel<uint16_t>, grid, block, lds, s, (const uint16_t*)x,
                       (const uint16_t*)router_w, bias, E, K, KS, d, norm_topk, idx, wpair, user_idx, user_w);
  return hipGetLastError();
}

}  // namespace moe
