// Expert SwiGLU FFN (paper section 2, Eq. 3) as a grouped bf16 GEMM on the
// CDNA4 matrix cores, for expert blocks in the tiled layout.
//
// Decode is weight-streaming: every (token, expert) pair moves 6*d*d_ff bytes
// of weights for 6*d*d_ff flops per token of the group, far below the
// machine's flop/byte ridge, so the kernels are organised around the weight
// stream and not around operand reuse:
//   * weights are the A operand of v_mfma_f32_16x16x32_bf16; the tiled layout
//     stores each 16-row x 32-column fragment as one contiguous 1 KiB run in
//     exactly the lane order of the instruction, so every wave-wide 16-byte
//     load is a fully coalesced 1 KiB request and no LDS staging or transpose
//     is needed for the weights;
//   * tokens are the B operand (up to 16 per MFMA column block), read straight
//     from L2 - they are a few KiB;
//   * a workgroup owns one 16-row output tile of one expert and its waves split
//     the contraction (split-K inside the workgroup), so even a single token
//     per expert yields thousands of waves each with a deep queue of loads;
//     partial tiles meet in LDS in a fixed order (deterministic sums).
// Phase 1 (NMAT = 2) computes h = silu(X W_g^T) * (X W_u^T) with gate and up
// fragments interleaved in memory; phase 2 (NMAT = 1) computes o = h W_d^T.
//
// Tiled layout of one expert block (bf16 elements, total 3*d*f):
//   [f/16 row tiles][d/32 k-blocks][gate,up][64 lanes][8]   then
//   [f/32 k-blocks][d/16 row tiles][64 lanes][8]
// with lane l, element j of a fragment holding W[row0 + l%16][k0 + (l/16)*8 + j].
#include "device_utils.hpp"
#include "moe_internal.hpp"

namespace moe {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// weights are read once per call: nontemporal, so that they do not displace the tokens, h and the router matrix
__device__ __forceinline__ uint4 ldw(const uint4* p) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return uint4{v.x, v.y, v.z, v.w};
}

__device__ __forceinline__ const char* group_weights(const FfnArgs& a, int id) {
  return id < a.P ? a.buffers + (size_t)id * a.expert_bytes
                  : a.shared + (size_t)(id - a.P) * a.expert_bytes;
}

template <int NMAT, int WAVES, int CH, int TT>
__global__ void __launch_bounds__(64 * WAVES) ffn_tiled_kernel(FfnArgs a) {
  __shared__ float red[WAVES][TT][NMAT][256];
  const int g = blockIdx.y;
  const int ng = *a.t.n_groups;        // both loads are issued before the first branch: one round trip
  const GroupDesc gd = a.t.grp[g];
  if (g >= ng || (a.pass != 2 && gd.miss != a.pass)) return;

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n = lane & 15;   // token column of the B operand / of the result
  const int q = lane >> 4;   // which 8-wide slice of the 32-deep k-block this lane feeds
  const int tile = blockIdx.x;
  const int kdim = NMAT == 2 ? a.d : a.f;   // contraction length
  const int nkb = kdim >> 5;
  const int kb0 = (int)((long)wave * nkb / WAVES), kb1 = (int)((long)(wave + 1) * nkb / WAVES);

  // fragment (tile, kb, m) of the gate/up section sits at ((tile*nkb + kb)*2 + m)*64 uint4;
  // fragment (tile, kb) of the down section at (kb*(d/16) + tile)*64 behind it
  const uint4* w = reinterpret_cast<const uint4*>(group_weights(a, gd.buf));
  size_t kb_stride;
  if (NMAT == 2) {
    w += (size_t)tile * nkb * 2 * 64 + lane;
    kb_stride = 2 * 64;
  } else {
    w += (size_t)2 * a.f * a.d / 8 + (size_t)tile * 64 + lane;
    kb_stride = (size_t)(a.d >> 4) * 64;
  }

  const int begin = gd.begin, cnt = gd.count;

  for (int tok0 = 0; tok0 < cnt; tok0 += 16 * TT) {
    const uint16_t* brow[TT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      const int tok = tok0 + tt * 16 + n;
      if (tok < cnt) {
        if (NMAT == 2) {
          const int p = a.t.sorted_pair[begin + tok];
          brow[tt] = reinterpret_cast<const uint16_t*>(a.x) + (size_t)(p / a.KS) * a.d + q * 8;
        } else {
          brow[tt] = reinterpret_cast<const uint16_t*>(a.h) + (size_t)(begin + tok) * a.f + q * 8;
        }
      } else {
        brow[tt] = nullptr;
      }
    }
    f32x4 acc[TT][NMAT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int m = 0; m < NMAT; ++m) acc[tt][m] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int kb = kb0; kb < kb1; kb += CH) {
      uint4 wf[CH][NMAT];
#pragma unroll
      for (int i = 0; i < CH; ++i)
#pragma unroll
        for (int m = 0; m < NMAT; ++m)
          wf[i][m] = (kb + i < kb1) ? ldw(w + (size_t)(kb + i) * kb_stride + m * 64) : uint4{0, 0, 0, 0};
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) {
        if (tok0 + tt * 16 < cnt) {   // uniform
#pragma unroll
          for (int i = 0; i < CH; ++i) {
            uint4 bv = uint4{0, 0, 0, 0};
            if (brow[tt] != nullptr && kb + i < kb1)
              bv = *reinterpret_cast<const uint4*>(brow[tt] + (size_t)(kb + i) * 32);
            const bf16x8 bfrag = __builtin_bit_cast(bf16x8, bv);
#pragma unroll
            for (int m = 0; m < NMAT; ++m)
              acc[tt][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[i][m]), bfrag,
                                                                   acc[tt][m], 0, 0, 0);
          }
        }
      }
    }

    // ---- partial tiles of the waves meet in LDS; summed in wave order ----
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
        *reinterpret_cast<f32x4*>(&red[wave][tt][m][lane * 4]) = acc[tt][m];
    __syncthreads();
    for (int el = threadIdx.x; el < TT * 256; el += 64 * WAVES) {
      const int tt = el >> 8, r = el & 255;
      const int nn = r >> 4, mm = r & 15;      // token column, row inside the tile
      const int tok = tok0 + tt * 16 + nn;
      if (tok < cnt) {
        // result element (row mm, column nn) sits in lane (mm/4)*16 + nn, register mm%4
        const int src = ((mm >> 2) * 16 + nn) * 4 + (mm & 3);
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int wv = 0; wv < WAVES; ++wv) {
          s0 += red[wv][tt][0][src];
          if (NMAT == 2) s1 += red[wv][tt][NMAT - 1][src];
        }
        if (NMAT == 2) {
          reinterpret_cast<uint16_t*>(a.h)[(size_t)(begin + tok) * a.f + tile * 16 + mm] =
              f32_to_bf16(silu(s0) * s1);
        } else {
          a.o[(size_t)(begin + tok) * a.d + tile * 16 + mm] = s0;
        }
      }
    }
    __syncthreads();
  }
}

}  // namespace

hipError_t launch_ffn_tiled(hipStream_t s, const FfnArgs& a, KernelEvents e1, KernelEvents e2) {
  if (a.g_max <= 0) return hipSuccess;
#ifndef MOE_FFN_WAVES
#define MOE_FFN_WAVES 8
#endif
#ifndef MOE_FFN_CH
#define MOE_FFN_CH 8
#endif
  constexpr int WAVES = MOE_FFN_WAVES, CH = MOE_FFN_CH;
  dim3 block(64 * WAVES);
  dim3 g1(a.f / 16, a.g_max), g2(a.d / 16, a.g_max);
  if (a.max_count <= 16) {
    launch_timed(ffn_tiled_kernel<2, WAVES, CH, 1>, g1, block, 0, s, e1, a);
    launch_timed(ffn_tiled_kernel<1, WAVES, CH, 1>, g2, block, 0, s, e2, a);
  } else {
    launch_timed(ffn_tiled_kernel<2, WAVES, CH, 2>, g1, block, 0, s, e1, a);
    launch_timed(ffn_tiled_kernel<1, WAVES, CH, 2>, g2, block, 0, s, e2, a);
  }
  return hipGetLastError();
}

}  // namespace moe
