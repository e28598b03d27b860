// Pieces of the routing and cache-lookup phases that more than one kernel uses: the gating of one token by one
// wave (paper Eq. 1 and the gate weights of Eq. 2) and the register-resident LRU table of a layer.
#pragma once
#include "device_utils.hpp"
#include "moe_internal.hpp"

namespace moe {

// ordering point between the lanes of ONE wave (LDS and global), no s_barrier
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
  __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ int readlane_i(int v, int lane) { return __builtin_amdgcn_readlane(v, lane); }

__device__ __forceinline__ int64_t uniform64(int64_t v) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

// The register-resident table: LRU, at most 64 slots and 64 buffers, and at most 128 buffer ids in all.
__host__ __device__ inline bool fast_table(int policy, int C, int P, int n_shared) {
  return policy == MOE_POLICY_LRU && C <= kWave && P <= kWave && P + n_shared <= 2 * kWave;
}

// ---------------------------------------------------------------- phase 2
// One wave gates one token from the logits in LDS (zs[E]).  kWeights = false: only the selected set (idx_g) is
// formed - same selection, no softmax - for callers that need to know which experts run, not their weights.
template <int EPL, bool kWeights = true>
__device__ __forceinline__ void gate_token(const float* zs, int b, int E, int K, int KS, int norm_topk,
                                           int32_t* idx_g, float* wpair_g, int32_t* user_idx, float* user_w,
                                           int32_t* idx_stage) {
  const int lane = threadIdx.x & 63;
  float z[EPL];
  bool sel[EPL];
  float zmax = -INFINITY;
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int e = lane + i * kWave;
    z[i] = e < E ? zs[e] : -INFINITY;
    sel[i] = false;
    zmax = fmaxf(zmax, z[i]);
  }
  zmax = wave_max(zmax);
  if (K <= 16) {
    // K rounds of arg-max; a taken entry is masked out; ties resolve to the lowest id
    float zc[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) zc[i] = z[i];
    for (int k = 0; k < K; ++k) {
      float m = zc[0];
#pragma unroll
      for (int i = 1; i < EPL; ++i) m = fmaxf(m, zc[i]);
      m = wave_max(m);
      bool done = false;
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        const uint64_t cand = __ballot(zc[i] == m && (lane + i * kWave) < E);
        if (!done && cand != 0) {          // uniform
          const int first = __ffsll((unsigned long long)cand) - 1;
          if (lane == first) { sel[i] = true; zc[i] = -INFINITY; }
          done = true;
        }
      }
    }
  } else {
    // rank every logit against all others (ties to the lower id)
    int rank[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) rank[i] = 0;
    for (int j = 0; j < E; ++j) {
      const float zj = zs[j];  // same address in every lane: LDS broadcast
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        const int e = lane + i * kWave;
        rank[i] += (zj > z[i] || (zj == z[i] && j < e)) ? 1 : 0;
      }
    }
#pragma unroll
    for (int i = 0; i < EPL; ++i) sel[i] = (lane + i * kWave) < E && rank[i] < K;
  }
  if constexpr (!kWeights) {
    int base = 0;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      const uint64_t m = __ballot(sel[i]);
      if (sel[i]) idx_g[(size_t)b * K + base + __popcll(m & ((1ull << lane) - 1ull))] = lane + i * kWave;
      base += __popcll(m);
    }
    return;
  }
  float p[EPL];
  float psum = 0.f;
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    p[i] = (lane + i * kWave) < E ? expf(z[i] - zmax) : 0.f;
    psum += p[i];
  }
  psum = wave_sum(psum);
  float selsum = 0.f;
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    p[i] = p[i] / psum;
    selsum += sel[i] ? p[i] : 0.f;
  }
  selsum = wave_sum(selsum);
  int base = 0;
#pragma unroll
  for (int i = 0; i < EPL; ++i) {
    const int e = lane + i * kWave;
    const uint64_t m = __ballot(sel[i]);
    if (sel[i]) {
      const int pos = base + __popcll(m & ((1ull << lane) - 1ull));   // ascending expert id
      const float w = norm_topk ? p[i] / selsum : p[i];
      idx_g[(size_t)b * K + pos] = e;
      wpair_g[(size_t)b * KS + pos] = w;
      if (idx_stage) idx_stage[(size_t)b * K + pos] = e;
      if (user_idx) user_idx[(size_t)b * K + pos] = e;
      if (user_w) user_w[(size_t)b * K + pos] = w;
    }
    base += __popcll(m);
  }
  if (lane < KS - K) wpair_g[(size_t)b * KS + K + lane] = 1.0f;  // shared experts: weight 1
}

// ---------------------------------------------------------------- phase 3, register path
// LRU with at most 64 slots, 64 buffers and 64 (token, expert) pairs: lane s holds
// slot s (expert, last-use tick, buffer), lane p holds buffer p's use stamp, lane i
// holds entry i of the free and released-buffer stacks, lane q holds pair q.
struct FastTable {
  int exp, buf, free_b, zomb;
  uint64_t tick;
  uint32_t used;
  int64_t clock, trace_n;
  int n_res, n_free, n_zombie;
};

__device__ __forceinline__ FastTable fast_load(const LayerState& st, int C, int P) {
  const int lane = threadIdx.x & 63;
  FastTable f;
  // the scalars are the same in every lane; telling the compiler so keeps the loops over them and the
  // cross-lane reads indexed by them on the scalar unit
  f.clock = uniform64(st.scalars[SC_CLOCK]);
  f.n_res = __builtin_amdgcn_readfirstlane((int)st.scalars[SC_NRES]);
  f.n_free = __builtin_amdgcn_readfirstlane((int)st.scalars[SC_NFREE]);
  f.n_zombie = __builtin_amdgcn_readfirstlane((int)st.scalars[SC_NZOMBIE]);
  f.trace_n = uniform64(st.scalars[SC_TRACE_N]);
  f.exp = lane < C ? st.expert_in[lane] : -2;
  f.tick = lane < C ? st.tick[lane] : ~0ull;
  f.buf = lane < C ? st.buf_of_slot[lane] : -1;
  f.used = lane < P ? st.used_stamp[lane] : 0u;
  f.free_b = lane < P ? st.free_buf[lane] : -1;
  f.zomb = lane < P ? st.zombie[lane] : -1;
  return f;
}

// index of the lane (< C) holding the smallest tick; ticks of valid lanes are unique
__device__ __forceinline__ int wave_argmin_tick(uint64_t tick) {
  uint32_t hi = (uint32_t)(tick >> 32), lo = (uint32_t)tick;
#define MOE_MIN_STEP(CTRL)                                                                              \
  {                                                                                                     \
    const uint32_t ohi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)hi, CTRL, 0xf, 0xf, true);       \
    const uint32_t olo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lo, CTRL, 0xf, 0xf, true);       \
    const bool less = ohi < hi || (ohi == hi && olo < lo);                                              \
    hi = less ? ohi : hi;                                                                               \
    lo = less ? olo : lo;                                                                               \
  }
  MOE_MIN_STEP(0xB1) MOE_MIN_STEP(0x4E) MOE_MIN_STEP(0x141) MOE_MIN_STEP(0x140)
#undef MOE_MIN_STEP
  uint64_t best = ~0ull;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const uint64_t v = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)hi, r * 16) << 32) |
                       (uint32_t)__builtin_amdgcn_readlane((int)lo, r * 16);
    best = v < best ? v : best;
  }
  return __ffsll((unsigned long long)__ballot(tick == best)) - 1;
}

}  // namespace moe
