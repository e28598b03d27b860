// Decode-shape expert FFN (paper section 2, Eq. 3) on INT4 group-quantised
// experts (section 3.2: experts are kept in 4-bit form so that more of them fit
// the cache and a miss moves a quarter of the bytes), in one launch.
//
// Format: every matrix is cut into groups of 32 consecutive elements along its
// contraction dimension; a group stores 32 4-bit codes q in 0..15 and one bf16
// scale s, and stands for the weights s * (q - 8) (4.5 bits per weight).
//
// Same decomposition as the bf16 kernel (ffn_fused.hip): a workgroup owns one
// expert and one chunk of 32 rows of the intermediate dimension; phase A
// computes h of the chunk (2 row tiles x waves/2 contraction slices, LDS
// reduction), phase B multiplies the chunk's k-block of W_d and writes partial
// rows [pair][chunk][d], summed later by combine_chunks_kernel.
//
// Dequantisation rides on the matrix cores:
//   * a code becomes the bf16 number 128 + q by OR-ing it into the mantissa of
//     0x4300 (two codes per 32-bit operation);
//   * tokens are the A operand and weights the B operand of
//     v_mfma_f32_16x16x32_bf16, so a lane ends up with one weight row (column of
//     D) for four tokens and needs ONE scale per k-block;
//   * one extra MFMA per k-block with the constant -136 as B operand yields
//     -136 * sum_k x_k for every token; used as the C input of the weight MFMAs
//     it turns sum (128 + q) x into sum (q - 8) x.  One k-block = one group, so
//     the result is multiplied by the group's scale and accumulated in fp32.
// A 16-byte load per lane covers four k-blocks (gate/up) or four row tiles
// (W_d), so loads stay one KiB per wave instruction as in the bf16 kernel.
#include "device_utils.hpp"
#include "moe_internal.hpp"
#include "q4_layout.hpp"
#include "routed_prologue.hpp"

namespace moe {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Items a wave keeps in flight.  Shallow on purpose: the unpacked operands and the MFMA chains of four k-blocks
// already take ~100 registers, and staying under 128 lets two workgroups share a compute unit, which hides the
// start-up and the LDS reduction of one behind the streaming of the other (measured: 64 -> 47 us on the
// Mixtral-like shape against rings of 4 and 8).
constexpr int kDepthA = 1;   // gate/up items (2.25 KiB each)
constexpr int kDepthB = 4;   // W_d items (1.125 KiB each)

template <typename V>
__device__ __forceinline__ V ldnt(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const V*>(p));
}

// eight codes of one 32-bit word -> eight bf16 values 128 + q; element 2p sits in nibble p, element 2p+1 in nibble 4+p
__device__ __forceinline__ bf16x8 codes_to_bf16(uint32_t w) {
  u32x4 r;
  r[0] = (w & 0x000F000Fu) | 0x43004300u;
  r[1] = ((w >> 4) & 0x000F000Fu) | 0x43004300u;
  r[2] = ((w >> 8) & 0x000F000Fu) | 0x43004300u;
  r[3] = ((w >> 12) & 0x000F000Fu) | 0x43004300u;
  return __builtin_bit_cast(bf16x8, r);
}

// bf16 element e of a packed register array, widened
template <typename V>
__device__ __forceinline__ float scale_at(V v, int e) {
  const uint32_t dw = v[e >> 1];
  return __uint_as_float((e & 1) ? (dw & 0xFFFF0000u) : (dw << 16));
}

__device__ __forceinline__ const char* group_weights(const FfnArgs& a, int id) {
  return id < a.P ? a.buffers + (size_t)id * a.expert_bytes
                  : a.shared + (size_t)(id - a.P) * a.expert_bytes;
}

// ONE: every group holds a single token (batch 1).  Only component 0 of the MFMA results (token 0 of the tile) is
// then scaled and accumulated, which removes a quarter of the vector arithmetic that bounds this kernel.
// ROUTED: the launch is the decode call up to the combine; every workgroup first derives the routing, the cache
// lookups and the groups for itself (routed_prologue.hpp).
template <int WAVES, bool ONE, bool ROUTED>
__device__ __forceinline__ void fused_q4_body(const FfnArgs& a, const RoutedArgs* rap) {
  __shared__ float red[WAVES][2][256];            // partial gate / up tiles of the waves
  __shared__ __align__(16) uint16_t hs[16][32];   // h of the chunk, bf16, [token][row in chunk]
  __shared__ typename std::conditional<ROUTED, RoutedLds, int>::type rl_store;
  GroupView gd;
  int pair0 = 0;
  if constexpr (ROUTED) {
    if (!routed_prologue<WAVES>(a, *rap, rl_store, &red[0][0][0], gd)) return;
  } else {
    const int g = blockIdx.y;
    const int ng = *a.t.n_groups;
    const GroupDesc gdg = a.t.grp[g];
    if (g >= ng || (a.pass != 2 && gdg.miss != a.pass)) return;
    gd.buf = gdg.buf; gd.begin = gdg.begin; gd.count = gdg.count; gd.miss = gdg.miss; gd.expert = gdg.expert;
    pair0 = gdg.pair0;
  }

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: the same in all lanes of a wave
  const int n = lane & 15;   // A operand: token row; B operand and D: weight row (column of D)
  const int q = lane >> 4;   // operands: 8-wide slice of the k-block; D: tokens 4q .. 4q+3
  const int c = blockIdx.x;  // chunk of 32 intermediate rows
  const int d = a.d;
  const int nsb = d >> 7;    // super-blocks of 128 along d_model
  const int n_dq = d >> 6;   // blocks of 64 rows of W_d
  constexpr int KS = WAVES / 2;
  const int tile = wave & 1, ks = wave >> 1;
  const int na = nsb / KS;        // gate/up items of this wave   (host guarantees divisibility)
  const int nb = n_dq / WAVES;    // W_d items of this wave

  const bool from_host = a.fetch != 0 && gd.miss != 0;
  const char* wdev = group_weights(a, gd.buf);
  const char* wsrc = from_host ? a.pool + (size_t)gd.expert * a.expert_bytes : wdev;
  const intptr_t fill_delta = reinterpret_cast<intptr_t>(wdev) - reinterpret_cast<intptr_t>(wsrc);
  auto fill = [&](const char* src, auto v) {     // same offset inside the device block
    *reinterpret_cast<decltype(v)*>(reinterpret_cast<intptr_t>(src) + fill_delta) = v;
  };
  // items are dealt round-robin: the waves of a workgroup read adjacent records at any moment
  const char* pa = wsrc + ((size_t)(2 * c + tile) * nsb + ks) * q4::kGateUpRecord;
  const char* pb = wsrc + q4::gate_up_bytes(d, a.f) + ((size_t)c * n_dq + wave) * q4::kDownRecord;
  constexpr size_t a_step = (size_t)KS * q4::kGateUpRecord, b_step = (size_t)WAVES * q4::kDownRecord;

  const int begin = gd.begin, cnt = gd.count;
  const uint16_t* xrow = nullptr;
  if (n < cnt) {
    int p;
    if constexpr (ROUTED) p = rl_store.sorted_pair[begin + n];
    else p = n == 0 ? pair0 : a.t.sorted_pair[begin + n];
    xrow = reinterpret_cast<const uint16_t*>(a.x) + (size_t)(p / a.KS) * d + (size_t)ks * 128 + q * 8;
  }

  u32x4 awg[kDepthA], awu[kDepthA], asc[kDepthA], ax[kDepthA][4];
  u32x4 bwd[kDepthB];
  u32x2 bsd[kDepthB];
  auto issue_a = [&](int slot, int item) {
    if (item < na) {
      const char* rec = pa + (size_t)item * a_step;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        ax[slot][j] = xrow ? *reinterpret_cast<const u32x4*>(xrow + (size_t)item * (KS * 128) + j * 32)
                           : u32x4{0, 0, 0, 0};
      awg[slot] = ldnt<u32x4>(rec + lane * 16);
      awu[slot] = ldnt<u32x4>(rec + 1024 + lane * 16);
      asc[slot] = ldnt<u32x4>(rec + 2048 + n * 16);
    }
  };
  auto issue_b = [&](int slot, int item) {
    if (item < nb) {
      const char* rec = pb + (size_t)item * b_step;
      bwd[slot] = ldnt<u32x4>(rec + lane * 16);
      bsd[slot] = ldnt<u32x2>(rec + 1024 + n * 8);
    }
  };
#pragma unroll
  for (int u = 0; u < kDepthA; ++u) issue_a(u, u);
#pragma unroll
  for (int u = 0; u < kDepthB; ++u) issue_b(u, u);

  const bf16x8 minus136 = __builtin_bit_cast(bf16x8, u32x4{0xC308C308u, 0xC308C308u, 0xC308C308u, 0xC308C308u});
  const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
  f32x4 accg = zero, accu = zero;
  for (int base = 0; base < na; base += kDepthA) {
#pragma unroll
    for (int u = 0; u < kDepthA; ++u) {
      if (base + u < na) {      // uniform
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bf16x8 xa = __builtin_bit_cast(bf16x8, ax[u][j]);
          const f32x4 off = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, minus136, zero, 0, 0, 0);
          const f32x4 dg = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, codes_to_bf16(awg[u][j]), off, 0, 0, 0);
          const f32x4 du = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xa, codes_to_bf16(awu[u][j]), off, 0, 0, 0);
          if (ONE) {
            accg[0] = fmaf(scale_at(asc[u], j), dg[0], accg[0]);
            accu[0] = fmaf(scale_at(asc[u], 4 + j), du[0], accu[0]);
          } else {
            accg += scale_at(asc[u], j) * dg;
            accu += scale_at(asc[u], 4 + j) * du;
          }
        }
        if (from_host) {
          const char* rec = pa + (size_t)(base + u) * a_step;
          fill(rec + lane * 16, awg[u]);
          fill(rec + 1024 + lane * 16, awu[u]);
          if (q == 0) fill(rec + 2048 + n * 16, asc[u]);
        }
        issue_a(u, base + u + kDepthA);
      }
    }
  }

  // ---- h of the chunk: the contraction slices of each row tile meet in LDS ----
  *reinterpret_cast<f32x4*>(&red[wave][0][lane * 4]) = accg;
  *reinterpret_cast<f32x4*>(&red[wave][1][lane * 4]) = accu;
  __syncthreads();
  for (int el = threadIdx.x; el < 512; el += 64 * WAVES) {
    const int tl = el >> 8, r = el & 255;
    const int nn = r >> 4, mm = r & 15;                         // token, row inside the tile
    const int src = ((nn >> 2) * 16 + mm) * 4 + (nn & 3);       // where the MFMA left element (token nn, row mm)
    float vg = 0.f, vu = 0.f;
#pragma unroll
    for (int k = 0; k < KS; ++k) {
      vg += red[k * 2 + tl][0][src];
      vu += red[k * 2 + tl][1][src];
    }
    hs[nn][tl * 16 + mm] = nn < cnt ? f32_to_bf16(silu(vg) * vu) : (uint16_t)0;
  }
  __syncthreads();

  // ---- phase B: W_d[:, chunk] h; the chunk is the only k-block (= one group), so every result is final ----
  const bf16x8 hb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(&hs[n][q * 8]));
  const f32x4 hoff = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hb, minus136, zero, 0, 0, 0);
  const size_t n_chunks = (size_t)(a.f >> 5);
  // lane: rows 64 dq + 4n .. +3 of W_d (one per register of the load) for tokens 4q .. 4q+3
  float* obase = a.o + ((size_t)(begin + q * 4) * n_chunks + c) * d + n * 4;
  for (int base = 0; base < nb; base += kDepthB) {
#pragma unroll
    for (int u = 0; u < kDepthB; ++u) {
      const int j = base + u;
      if (j < nb) {             // uniform
        f32x4 r[4] = {zero, zero, zero, zero};
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          const f32x4 dd = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hb, codes_to_bf16(bwd[u][m]), hoff, 0, 0, 0);
          if (ONE) r[m][0] = scale_at(bsd[u], m) * dd[0];
          else r[m] = scale_at(bsd[u], m) * dd;
        }
        if (from_host) {
          const char* rec = pb + (size_t)j * b_step;
          fill(rec + lane * 16, bwd[u]);
          if (q == 0) fill(rec + 1024 + n * 8, bsd[u]);
        }
        issue_b(u, j + kDepthB);
        const int dq = wave + WAVES * j;
#pragma unroll
        for (int i = 0; i < (ONE ? 1 : 4); ++i)
          if (q * 4 + i < cnt)
            *reinterpret_cast<f32x4*>(obase + (size_t)i * n_chunks * d + (size_t)dq * 64) =
                f32x4{r[0][i], r[1][i], r[2][i], r[3][i]};
      }
    }
  }
}

template <int WAVES, bool ONE>
__global__ void __launch_bounds__(64 * WAVES) ffn_fused_q4_kernel(FfnArgs a) {
  fused_q4_body<WAVES, ONE, false>(a, nullptr);
}

template <int WAVES, bool ONE>
__global__ void __launch_bounds__(64 * WAVES, 4) decode_single_q4_kernel(FfnArgs a, RoutedArgs ra) {
  fused_q4_body<WAVES, ONE, true>(a, &ra);
}

int pick_waves_q4(int d) { return d % 512 == 0 ? 8 : d % 256 == 0 ? 4 : 0; }

}  // namespace

bool ffn_fused_q4_supported(int d, int f, int max_count) {
  return max_count <= 16 && f % 32 == 0 && d >= 256 && pick_waves_q4(d) != 0;
}

int fused_q4_waves(int d) { return pick_waves_q4(d); }

hipError_t launch_decode_single_q4(hipStream_t s, const FfnArgs& a, const RoutedArgs& ra, KernelEvents ev) {
  dim3 grid(a.f / 32, a.g_max + 1);     // + the bookkeeping row
  switch (pick_waves_q4(a.d)) {
    case 8:
      if (a.max_count == 1) launch_timed(decode_single_q4_kernel<8, true>, grid, dim3(512), 0, s, ev, a, ra);
      else launch_timed(decode_single_q4_kernel<8, false>, grid, dim3(512), 0, s, ev, a, ra);
      break;
    case 4:
      if (a.max_count == 1) launch_timed(decode_single_q4_kernel<4, true>, grid, dim3(256), 0, s, ev, a, ra);
      else launch_timed(decode_single_q4_kernel<4, false>, grid, dim3(256), 0, s, ev, a, ra);
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_ffn_fused_q4(hipStream_t s, const FfnArgs& a, KernelEvents ev) {
  if (a.g_max <= 0) return hipSuccess;
  dim3 grid(a.f / 32, a.g_max);
  switch (pick_waves_q4(a.d)) {
    case 8:
      if (a.max_count == 1) launch_timed(ffn_fused_q4_kernel<8, true>, grid, dim3(512), 0, s, ev, a);
      else launch_timed(ffn_fused_q4_kernel<8, false>, grid, dim3(512), 0, s, ev, a);
      break;
    case 4:
      if (a.max_count == 1) launch_timed(ffn_fused_q4_kernel<4, true>, grid, dim3(256), 0, s, ev, a);
      else launch_timed(ffn_fused_q4_kernel<4, false>, grid, dim3(256), 0, s, ev, a);
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace moe
