// Cache-simulation loss over routing traces (paper section 3.1.1; appendix C.1,
// Definition C.1 and Proposition C.2): forward value of the soft loss L_cs and
// of the hard miss count L_cs^hard.
//
// The recursion over tokens is sequential, so one workgroup walks one trace
// (one layer of one sequence) with one thread per expert: the soft state c_e
// and the discounted count Ctilde_e live in a register each.  Per token the
// owners of the K requested experts publish their two values to LDS; every
// thread ranks its count against them (wave ballots + LDS adds), which gives
// Top-C membership of the requested experts without sorting; thread 0 adds the
// K terms in request order.  Traces run in parallel across workgroups.  All
// arithmetic is fp64 without contraction, in the order the recursion is
// written, so the Top-C decisions agree with a plain CPU evaluation.  With at most 64 experts a single wave does
// the same without LDS or barriers (cache_sim_wave_kernel below).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe_cache.h"
#include "moe_internal.hpp"

namespace {

constexpr int kSimMaxK = 64;

#pragma clang fp contract(off)
__global__ void __launch_bounds__(1024) cache_sim_kernel(const int32_t* __restrict__ idx, int T, int K, int E, int C,
                                                         double gamma, const double* __restrict__ c1,
                                                         double* __restrict__ out, int32_t* __restrict__ bad) {
  __shared__ double sh_c[2][kSimMaxK], sh_ct[2][kSimMaxK];
  __shared__ int sh_rank[2][kSimMaxK];
  const int trace = blockIdx.x;
  const int e = threadIdx.x;
  const int lane = threadIdx.x & 63;
  const bool live = e < E;
  const int32_t* r = idx + (size_t)trace * T * K;
  double c = live ? (c1 ? c1[(size_t)trace * E + e] : (double)C / (double)E) : 0.0;
  double ct = c;
  double Gamma = 1.0, soft = 0.0, hard = 0.0;
  const double k_over_c = (double)K / (double)C;
  if (e < 2 * kSimMaxK) (&sh_rank[0][0])[e] = 0;
  for (int i = e + blockDim.x; i < 2 * kSimMaxK; i += blockDim.x) (&sh_rank[0][0])[i] = 0;
  int invalid = 0;
  __syncthreads();
  for (int t = 0; t < T; ++t) {
    const int p = t & 1;
    const int32_t* rt = r + (size_t)t * K;
    for (int k = 0; k < K; ++k) {
      const int rk = rt[k];
      if (rk == e) { sh_c[p][k] = c; sh_ct[p][k] = ct; }
      if (rk < 0 || rk >= E) invalid = 1;
    }
    if (invalid) break;                       // uniform: every thread reads the same ids
    __syncthreads();
    for (int k = 0; k < K; ++k) {
      const int rk = rt[k];
      const double v = sh_ct[p][k];
      const bool ahead = live && (ct > v || (ct == v && e < rk));
      const unsigned long long m = __ballot(ahead);
      if (lane == 0 && m) atomicAdd(&sh_rank[p][k], __popcll(m));
    }
    __syncthreads();
    if (e == 0) {
      for (int k = 0; k < K; ++k) {
        soft += 1.0 - sh_c[p][k];
        hard += sh_rank[p][k] < C ? 0.0 : 1.0;
        sh_rank[p][k] = 0;                    // this parity is ranked again two tokens later, after two barriers
      }
    }
    const double Gamma_next = gamma * Gamma + k_over_c;
    double cn = gamma * Gamma * c;
    double ctn = gamma * ct;
    for (int k = 0; k < K; ++k)
      if (rt[k] == e) { cn += 1.0; ctn += 1.0; }
    c = cn / Gamma_next;
    ct = ctn;
    Gamma = Gamma_next;
  }
  if (e == 0) {
    out[2 * trace] = soft;
    out[2 * trace + 1] = hard;
    bad[trace] = invalid;
  }
}

// Up to 64 experts: one wave walks the trace, lane e holding expert e.  The values of the requested experts are read
// with cross-lane moves (the requested id is wave-uniform), the rank is one ballot, and every lane carries the two
// sums, so a token step needs neither LDS nor a barrier; the ids of the next token are fetched while the current one
// is worked on.  Same arithmetic in the same order as the kernel above.
__device__ __forceinline__ double readlane_f64(double v, int lane) {
  const int hi = __builtin_amdgcn_readlane(__double2hiint(v), lane);
  const int lo = __builtin_amdgcn_readlane(__double2loint(v), lane);
  return __hiloint2double(hi, lo);
}

__global__ void __launch_bounds__(64) cache_sim_wave_kernel(const int32_t* __restrict__ idx, int T, int K, int E, int C,
                                                            double gamma, const double* __restrict__ c1,
                                                            double* __restrict__ out, int32_t* __restrict__ bad) {
  const int trace = blockIdx.x;
  const int lane = threadIdx.x;
  const bool live = lane < E;
  const int32_t* r = idx + (size_t)trace * T * K;
  double c = live ? (c1 ? c1[(size_t)trace * E + lane] : (double)C / (double)E) : 0.0;
  double ct = c;
  double Gamma = 1.0, soft = 0.0, hard = 0.0;
  const double k_over_c = (double)K / (double)C;
  int invalid = 0;
  int ids_next = (T > 0 && lane < K) ? r[lane] : 0;
  for (int t = 0; t < T; ++t) {
    const int ids = ids_next;                       // lane k: the k-th requested expert of token t
    if (t + 1 < T && lane < K) ids_next = r[(size_t)(t + 1) * K + lane];
    if (__ballot(lane < K && (ids < 0 || ids >= E)) != 0) { invalid = 1; break; }
    int mine = 0;                                   // times this lane's expert is requested by the token
    for (int k = 0; k < K; ++k) {
      const int rk = __builtin_amdgcn_readlane(ids, k);
      const double v = readlane_f64(ct, rk);
      const bool ahead = live && (ct > v || (ct == v && lane < rk));
      const int rank = __popcll(__ballot(ahead));
      soft += 1.0 - readlane_f64(c, rk);
      hard += rank < C ? 0.0 : 1.0;
      mine += lane == rk ? 1 : 0;
    }
    const double Gamma_next = gamma * Gamma + k_over_c;
    double cn = gamma * Gamma * c;
    double ctn = gamma * ct;
    for (int h = 0; h < mine; ++h) { cn += 1.0; ctn += 1.0; }
    c = cn / Gamma_next;
    ct = ctn;
    Gamma = Gamma_next;
  }
  if (lane == 0) {
    out[2 * trace] = soft;
    out[2 * trace + 1] = hard;
    bad[trace] = invalid;
  }
}

}  // namespace

extern "C" int moe_cache_sim_loss(const int32_t* idx_dev, int32_t n_traces, int32_t T, int32_t K, int32_t n_experts,
                                  int32_t capacity, double gamma, const double* c1_dev, double* out_dev,
                                  int32_t* flag_dev, void* hip_stream) {
  using moe::fail;
  if (n_traces < 0 || T < 0) return fail(MOE_ERR_INVALID_ARG, "n_traces and T must be >= 0");
  if ((!idx_dev && n_traces > 0 && T > 0) || ((!out_dev || !flag_dev) && n_traces > 0))
    return fail(MOE_ERR_INVALID_ARG, "null idx, out or flag buffer");
  if (n_experts < 1 || n_experts > 1024) return fail(MOE_ERR_INVALID_ARG, "n_experts must be in 1..1024");
  if (K < 1 || K > kSimMaxK || K > n_experts) return fail(MOE_ERR_INVALID_ARG, "K must be in 1..min(n_experts,64)");
  if (capacity < 1 || capacity > n_experts) return fail(MOE_ERR_INVALID_ARG, "capacity must be in 1..n_experts");
  if (!(gamma >= 0.0 && gamma <= 1.0)) return fail(MOE_ERR_INVALID_ARG, "gamma must be in [0,1]");
  if (n_traces == 0) return MOE_OK;
  const int threads = ((n_experts + 63) / 64) * 64;
  if (n_experts <= 64)
    hipLaunchKernelGGL(cache_sim_wave_kernel, dim3((unsigned)n_traces), dim3(64), 0,
                       static_cast<hipStream_t>(hip_stream), idx_dev, T, K, n_experts, capacity, gamma, c1_dev, out_dev,
                       flag_dev);
  else
    hipLaunchKernelGGL(cache_sim_kernel, dim3((unsigned)n_traces), dim3(threads), 0,
                       static_cast<hipStream_t>(hip_stream), idx_dev, T, K, n_experts, capacity, gamma, c1_dev, out_dev,
                       flag_dev);
  const hipError_t err = hipGetLastError();
  if (err != hipSuccess) return fail(MOE_ERR_HIP, "cache_sim_kernel launch: %s", hipGetErrorString(err));
  return MOE_OK;
}
