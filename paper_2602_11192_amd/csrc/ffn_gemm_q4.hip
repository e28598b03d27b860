// Expert SwiGLU FFN (paper section 2, Eq. 3) on INT4 group-quantised experts
// (section 3.2) as a grouped GEMM, for calls in which an expert sees many
// tokens: batched decode beyond 16 tokens and prompt processing.
//
// One workgroup = 4 waves x a tile of up to 64 of one expert's tokens.  Tokens
// are the A operand of v_mfma_f32_16x16x32_bf16, staged through LDS in fragment
// order, four k-blocks (128 columns) per step, double buffered; weights are the
// B operand, unpacked from 4-bit codes in registers (see ffn_fused_q4.hip for
// the 128 + q mantissa trick and the -136 correction fed through the C input).
// A lane holds one weight row for four tokens, so the per-group scale is one
// multiplier per k-block.
//   gate/up pass: wave w owns row tile 4 bx + w; one 16-byte load per lane
//     brings the codes of four k-blocks of W_g, another those of W_u, a third
//     the eight scales.  h = silu(g) * u is written as bf16, rows in group order.
//   down pass: wave w owns the block of 64 rows 4 bx + w of W_d; per k-block one
//     16-byte load per lane brings the codes of its four row tiles.
// Every weight byte is read by exactly one wave, so a group whose expert is not
// resident can stream it from the pinned host pool (prompt streaming).
#include "device_utils.hpp"
#include "moe_internal.hpp"
#include "q4_layout.hpp"

namespace moe {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 4;
constexpr int kSkb = 4;             // k-blocks staged per step

template <typename V>
__device__ __forceinline__ V ldnt(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const V*>(p));
}

__device__ __forceinline__ bf16x8 codes_to_bf16(uint32_t w) {
  u32x4 r;
  r[0] = (w & 0x000F000Fu) | 0x43004300u;
  r[1] = ((w >> 4) & 0x000F000Fu) | 0x43004300u;
  r[2] = ((w >> 8) & 0x000F000Fu) | 0x43004300u;
  r[3] = ((w >> 12) & 0x000F000Fu) | 0x43004300u;
  return __builtin_bit_cast(bf16x8, r);
}

template <typename V>
__device__ __forceinline__ float scale_at(V v, int e) {
  const uint32_t dw = v[e >> 1];
  return __uint_as_float((e & 1) ? (dw & 0xFFFF0000u) : (dw << 16));
}

__device__ __forceinline__ const char* group_weights(const FfnArgs& a, int id) {
  return id < a.P ? a.buffers + (size_t)id * a.expert_bytes
                  : a.shared + (size_t)(id - a.P) * a.expert_bytes;
}

// kTok: tokens per workgroup (64 or 128).  An expert streamed from the host is read once per token tile, so prompt
// streaming takes the large tile; the small one needs half the accumulators and serves every resident call.
template <int NMAT, int kTok>
__global__ void __launch_bounds__(64 * kWaves) ffn_gemm_q4_kernel(FfnArgs a) {
  constexpr int kCb = kTok / 16;      // column blocks of 16 tokens
  constexpr int kPieces = kTok / 16;  // 16-byte pieces of the token tile each thread stages per step
  // [buffer][k-block of the step][column block][lane] x 16 bytes
  __shared__ u32x4 xs[2][kSkb][kCb][64];
  const int g = blockIdx.y;
  const int ng = *a.t.n_groups;
  const GroupDesc gd = a.t.grp[g];
  if (g >= ng || (a.pass != 2 && gd.miss != a.pass)) return;
  const int tok0 = blockIdx.z * kTok;
  const int cnt = gd.count;
  if (tok0 >= cnt) return;
  const int n_tok = min(kTok, cnt - tok0);
  const int n_cb = (n_tok + 15) >> 4;

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n = lane & 15, q = lane >> 4;
  const int d = a.d, f = a.f;
  const int kdim = NMAT == 2 ? d : f;
  const int nkb = kdim >> 5;                                   // k-blocks of the contraction
  const int n_units = NMAT == 2 ? (f >> 4) : (d >> 6);         // row tiles of 16 / row blocks of 64
  const int unit = blockIdx.x * kWaves + wave;                 // this wave's row tile / row block
  const bool has_rows = unit < n_units;
  const int uc = has_rows ? unit : n_units - 1;                // clamped: loads stay in bounds, results are dropped

  const char* wsrc = (a.fetch != 0 && gd.miss != 0) ? a.pool + (size_t)gd.expert * a.expert_bytes
                                                    : group_weights(a, gd.buf);
  // gate/up: records [row tile][super-block of 4 k-blocks]; down: records [k-block][row block]
  const int nsb = d >> 7, n_dq = d >> 6;
  const char* wrec = NMAT == 2 ? wsrc + (size_t)uc * nsb * q4::kGateUpRecord
                               : wsrc + q4::gate_up_bytes(d, f) + (size_t)uc * q4::kDownRecord;

  // ---- token staging: 256 threads x kPieces pieces of 16 bytes = kTok rows x 256 bytes (4 k-blocks) ----
  const uint16_t* src[kPieces];
  int dst[kPieces];
#pragma unroll
  for (int i = 0; i < kPieces; ++i) {
    const int idx = threadIdx.x + 256 * i;
    const int r = idx >> 4, sg = idx & 15;                     // token row of the tile, 16-byte segment of its 256 bytes
    const int kbl = sg >> 2, qq = sg & 3;
    // the 16 lanes that write together hold one row's 16 (k-block, slice) pieces: the XOR spreads them over the banks
    dst[i] = (kbl * kCb + (r >> 4)) * 64 + qq * 16 + ((r & 15) ^ (qq + 4 * kbl));
    if (r < n_tok) {
      if (NMAT == 2) {
        const int p = a.t.sorted_pair[gd.begin + tok0 + r];
        src[i] = reinterpret_cast<const uint16_t*>(a.x) + (size_t)(p / a.KS) * d + sg * 8;
      } else {
        src[i] = reinterpret_cast<const uint16_t*>(a.h) + (size_t)(gd.begin + tok0 + r) * f + sg * 8;
      }
    } else {
      src[i] = nullptr;
    }
  }
  auto load_x = [&](u32x4 (&xr)[kPieces], int kb) {
#pragma unroll
    for (int i = 0; i < kPieces; ++i) {
      const int kbi = kb + ((threadIdx.x + 256 * i) & 15) / 4;   // k-block this piece belongs to
      xr[i] = (src[i] != nullptr && kbi < nkb) ? *reinterpret_cast<const u32x4*>(src[i] + (size_t)kb * 32)
                                                : u32x4{0, 0, 0, 0};
    }
  };
  // weights of one step: gate/up = codes of W_g, W_u and 8 scales of one super-block;
  //                      down    = codes of 4 row tiles and 4 scales for each of up to 4 k-blocks
  constexpr int NW = NMAT == 2 ? 3 : 6;
  auto load_w = [&](u32x4 (&wr)[NW], int kb) {
    if (NMAT == 2) {
      const char* rec = wrec + (size_t)(kb >> 2) * q4::kGateUpRecord;
      wr[0] = ldnt<u32x4>(rec + lane * 16);
      wr[1] = ldnt<u32x4>(rec + 1024 + lane * 16);
      wr[2] = ldnt<u32x4>(rec + 2048 + n * 16);
    } else {
#pragma unroll
      for (int j = 0; j < kSkb; ++j) {
        const int kbj = kb + j < nkb ? kb + j : nkb - 1;         // clamped; the surplus k-blocks are skipped below
        const char* rec = wrec + (size_t)kbj * n_dq * q4::kDownRecord;
        wr[j] = ldnt<u32x4>(rec + lane * 16);
        const u32x2 s2 = ldnt<u32x2>(rec + 1024 + n * 8);
        wr[4 + (j >> 1)][(j & 1) * 2] = s2[0];
        wr[4 + (j >> 1)][(j & 1) * 2 + 1] = s2[1];
      }
    }
  };

  const bf16x8 minus136 = __builtin_bit_cast(bf16x8, u32x4{0xC308C308u, 0xC308C308u, 0xC308C308u, 0xC308C308u});
  const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
  // gate/up: acc[cb][0] gate, acc[cb][1] up; down: acc[cb][j] row tile j of the block
  constexpr int NA = NMAT == 2 ? 2 : 4;
  f32x4 acc[kCb][NA];
#pragma unroll
  for (int cb = 0; cb < kCb; ++cb)
#pragma unroll
    for (int m = 0; m < NA; ++m) acc[cb][m] = zero;

  u32x4 xr[kPieces], wc[NW], wn[NW];
  load_x(xr, 0);
  load_w(wc, 0);
#pragma unroll
  for (int i = 0; i < kPieces; ++i) (&xs[0][0][0][0])[dst[i]] = xr[i];
  __syncthreads();

  int buf = 0;
  for (int kb = 0; kb < nkb; kb += kSkb) {
    const bool more = kb + kSkb < nkb;
    if (more) {
      load_x(xr, kb + kSkb);
      load_w(wn, kb + kSkb);
    }
#pragma unroll
    for (int j = 0; j < kSkb; ++j) {
      if (kb + j < nkb) {       // uniform
        bf16x8 wb[NA];
        float sc[NA];
        if (NMAT == 2) {
          wb[0] = codes_to_bf16(wc[0][j]);
          wb[1] = codes_to_bf16(wc[1][j]);
          sc[0] = scale_at(wc[2], j);
          sc[1] = scale_at(wc[2], 4 + j);
        } else {
#pragma unroll
          for (int m = 0; m < 4; ++m) {
            wb[m] = codes_to_bf16(wc[j][m]);
            sc[m] = scale_at(wc[4 + (j >> 1)], (j & 1) * 4 + m);
          }
        }
#pragma unroll
        for (int cb = 0; cb < kCb; ++cb) {
          if (cb < n_cb) {      // uniform
            const bf16x8 xa = __builtin_bit_cast(bf16x8, xs[buf][j][cb][lane ^ (q + 4 * j)]);
            const f32x4 off = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, minus136, zero, 0, 0, 0);
#pragma unroll
            for (int m = 0; m < NA; ++m)
              acc[cb][m] += sc[m] * __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, wb[m], off, 0, 0, 0);
          }
        }
      }
    }
    if (more) {
#pragma unroll
      for (int i = 0; i < kPieces; ++i) (&xs[buf ^ 1][0][0][0])[dst[i]] = xr[i];
#pragma unroll
      for (int m = 0; m < NW; ++m) wc[m] = wn[m];
    }
    __syncthreads();
    buf ^= 1;
  }

  // ---- epilogue: lane holds weight row n of its tile(s) for tokens 16 cb + 4 q + i ----
  if (!has_rows) return;
#pragma unroll
  for (int cb = 0; cb < kCb; ++cb) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int tk = cb * 16 + q * 4 + i;
      if (cb < n_cb && tk < n_tok) {
        const size_t pos = (size_t)(gd.begin + tok0 + tk);
        if (NMAT == 2) {
          reinterpret_cast<uint16_t*>(a.h)[pos * f + unit * 16 + n] =
              f32_to_bf16(silu(acc[cb][0][i]) * acc[cb][NA - 1][i]);
        } else {
          // rows 64 unit + 4 n + m, m = 0..3: one 16-byte store
          *reinterpret_cast<f32x4*>(a.o + pos * d + (size_t)unit * 64 + n * 4) =
              f32x4{acc[cb][0][i], acc[cb][1][i], acc[cb][NA > 2 ? 2 : 0][i], acc[cb][NA > 3 ? 3 : 0][i]};
        }
      }
    }
  }
}

}  // namespace

hipError_t launch_ffn_gemm_q4(hipStream_t s, const FfnArgs& a, KernelEvents e1, KernelEvents e2) {
  if (a.g_max <= 0) return hipSuccess;
  // 128-token tiles only when experts stream in from the host (each tile reads the expert over the link once).
  // On resident experts the 64-token tile is faster at every call size measured (OLMoE-like layer: 71 against
  // 127 us at 64 tokens per call, 280 against 413 us at 1024, 505 against 717 us at 2048): half the accumulators,
  // twice the workgroups per compute unit.
  const bool large_tile = a.fetch != 0;
  const int tok = large_tile ? 128 : 64;
  const int tiles = (a.max_count + tok - 1) / tok;
  dim3 block(64 * kWaves);
  dim3 g1((a.f / 16 + kWaves - 1) / kWaves, a.g_max, tiles);
  dim3 g2((a.d / 64 + kWaves - 1) / kWaves, a.g_max, tiles);
  if (large_tile) {
    launch_timed(ffn_gemm_q4_kernel<2, 128>, g1, block, 0, s, e1, a);
    launch_timed(ffn_gemm_q4_kernel<1, 128>, g2, block, 0, s, e2, a);
  } else {
    launch_timed(ffn_gemm_q4_kernel<2, 64>, g1, block, 0, s, e1, a);
    launch_timed(ffn_gemm_q4_kernel<1, 64>, g2, block, 0, s, e2, a);
  }
  return hipGetLastError();
}

}  // namespace moe
