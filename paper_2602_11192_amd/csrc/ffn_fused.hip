// Decode-shape expert FFN (paper section 2, Eq. 3) in ONE launch: gate/up
// projection, SiLU * up, and the down projection, for groups of at most 16
// tokens per expert (batch <= 16), on bf16 experts in the tiled layout.
//
// Why one launch: at decode an expert sees one or a few tokens, every weight
// byte is used once, and a whole layer call moves only ~100 MB - about 13 us of
// HBM time.  Two dependent kernels pay the launch ramp, the metadata round trip
// and the drain twice; here they are paid once.
//
// A workgroup owns one expert and one chunk of 32 rows of its intermediate
// dimension (one MFMA k-block of the down projection):
//   phase A: h[32 rows] = silu(W_g[rows,:] x) * (W_u[rows,:] x).  16 waves =
//     2 row tiles x 8 slices of the contraction; partial tiles meet in LDS.
//   phase B: partial o[:, d] = W_d[:, rows] h[rows]; each wave takes d/256 row
//     tiles of W_d; with the chunk as the only k-block every MFMA result is a
//     finished partial sum, written as [pair][chunk][d] fp32.
// The chunks of an expert are summed, in chunk order, by combine_chunks_kernel
// together with the gate-weighted sum over experts of Eq. 2 (deterministic).
//
// Each wave runs ONE software-pipelined stream over its fragments - first its
// gate/up fragments (with the matching token slices), then its W_d fragments -
// with up to kDepth fragments in flight; the W_d loads are already under way
// while the workgroup reduces h, so HBM never idles inside the workgroup.
#include "device_utils.hpp"
#include "moe_internal.hpp"

namespace moe {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kFusedWaves = 16;
constexpr int kDepth = 8;       // fragments (gate+up pairs count as one) a wave keeps in flight

__device__ __forceinline__ const char* group_weights(const FfnArgs& a, int g) {
  const int id = a.t.grp_buf[g];
  return id < a.P ? a.buffers + (size_t)id * a.expert_bytes
                  : a.shared + (size_t)(id - a.P) * a.expert_bytes;
}

// R = d / 256: k-blocks per wave in phase A and row tiles of W_d per wave in phase B.
template <int R>
__global__ void __launch_bounds__(64 * kFusedWaves) ffn_fused_kernel(FfnArgs a) {
  __shared__ float red[kFusedWaves][2][256];      // partial gate / up tiles of the 16 waves
  __shared__ __align__(16) uint16_t hs[16][32];   // h of the chunk, bf16, [token][row in chunk]
  const int g = blockIdx.y;
  if (g >= *a.t.n_groups) return;
  if (a.pass != 2 && a.t.grp_miss[g] != a.pass) return;

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n = lane & 15;   // token column
  const int q = lane >> 4;   // 8-wide slice of a 32-deep k-block
  const int c = blockIdx.x;  // chunk of 32 intermediate rows
  const int d = a.d;
  const int nkb_d = d >> 5, n_dt = d >> 4;
  const int tile = wave & 1, ks = wave >> 1;
  const int kb0 = ks * R;

  const uint4* wbase = reinterpret_cast<const uint4*>(group_weights(a, g));
  // gate/up fragment (row tile 2c+tile, kb, m) and W_d fragment (chunk c, row tile dt)
  const uint4* wa = wbase + ((size_t)(2 * c + tile) * nkb_d + kb0) * 2 * 64 + lane;
  const uint4* wb = wbase + (size_t)2 * a.f * d / 8 + ((size_t)c * n_dt + wave) * 64 + lane;

  const int begin = a.t.grp_begin[g], cnt = a.t.grp_count[g];
  const uint16_t* xrow = nullptr;
  if (n < cnt) {
    const int p = a.t.sorted_pair[begin + n];
    xrow = reinterpret_cast<const uint16_t*>(a.x) + (size_t)(p / a.KS) * d + (size_t)kb0 * 32 + q * 8;
  }

  // ---- one pipelined stream: R gate/up items, then R W_d items ----
  uint4 fg[R], fu[R], fx[R], fd[R];
  auto issue = [&](int i) {
    if (i < R) {
      fx[i] = xrow ? *reinterpret_cast<const uint4*>(xrow + (size_t)i * 32) : uint4{0, 0, 0, 0};
      fg[i] = wa[(size_t)i * 128];
      fu[i] = wa[(size_t)i * 128 + 64];
    } else {
      fd[i - R] = wb[(size_t)(i - R) * kFusedWaves * 64];
    }
  };
#pragma unroll
  for (int i = 0; i < kDepth && i < 2 * R; ++i) issue(i);

  f32x4 accg = {0.f, 0.f, 0.f, 0.f}, accu = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < R; ++i) {
    const bf16x8 xb = __builtin_bit_cast(bf16x8, fx[i]);
    accg = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fg[i]), xb, accg, 0, 0, 0);
    accu = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fu[i]), xb, accu, 0, 0, 0);
    if (i + kDepth < 2 * R) issue(i + kDepth);
  }

  // ---- h of the chunk: the 8 contraction slices of each row tile meet in LDS ----
  *reinterpret_cast<f32x4*>(&red[wave][0][lane * 4]) = accg;
  *reinterpret_cast<f32x4*>(&red[wave][1][lane * 4]) = accu;
  __syncthreads();
  if (threadIdx.x < 512) {
    const int tl = threadIdx.x >> 8, r = threadIdx.x & 255;
    const int nn = r >> 4, mm = r & 15;                         // token, row inside the tile
    const int src = ((mm >> 2) * 16 + nn) * 4 + (mm & 3);       // where the MFMA left element (mm, nn)
    float sg = 0.f, su = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      sg += red[k * 2 + tl][0][src];
      su += red[k * 2 + tl][1][src];
    }
    hs[nn][tl * 16 + mm] = nn < cnt ? f32_to_bf16(silu(sg) * su) : (uint16_t)0;
  }
  __syncthreads();

  // ---- phase B: W_d[:, chunk] h, R row tiles of 16 per wave ----
  const bf16x8 hb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&hs[n][q * 8]));
  const size_t n_chunks = (size_t)(a.f >> 5);
  float* obase = a.o + ((size_t)(begin + n) * n_chunks + c) * d + (lane >> 4) * 4;
#pragma unroll
  for (int j = 0; j < R; ++j) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fd[j]), hb, acc, 0, 0, 0);
    if (j + kDepth < R) issue(R + j + kDepth);   // only when R > kDepth
    // lane holds rows (lane/16)*4 .. +3 of row tile (wave + 16 j) for token n
    if (n < cnt) *reinterpret_cast<f32x4*>(obase + (size_t)(wave + kFusedWaves * j) * 16) = acc;
  }
}

// y[b][i] = sum_j wpair[b][j] * sum_c o_part[pos_of[b][j]][c][i].
// A workgroup owns 32 columns of one token; its 32 slices split the KS * n_chunks
// terms (every load issued before the first use), then the slices are summed in
// slice order: the result does not depend on timing.
constexpr int kCombCols = 32, kCombSlices = 32, kCombItems = 8;

template <typename T>
__global__ void __launch_bounds__(kCombCols * kCombSlices)
combine_chunks_kernel(const float* __restrict__ o_part, const float* __restrict__ wpair,
                      const int32_t* __restrict__ pos_of, int KS, int d, int n_chunks, T* __restrict__ y) {
  __shared__ float part[kCombSlices][kCombCols];
  const int b = blockIdx.x;
  const int col = threadIdx.x % kCombCols, sl = threadIdx.x / kCombCols;
  const int i = blockIdx.y * kCombCols + col;
  const int n_items = KS * n_chunks;
  const int per = (n_items + kCombSlices - 1) / kCombSlices;
  float acc = 0.f;
  if (i < d) {
    for (int it0 = sl * per; it0 < min((sl + 1) * per, n_items); it0 += kCombItems) {
      float v[kCombItems], w[kCombItems];
#pragma unroll
      for (int u = 0; u < kCombItems; ++u) {
        const int it = it0 + u;
        const bool ok = it < min((sl + 1) * per, n_items);
        const int j = ok ? it / n_chunks : 0, c = ok ? it - j * n_chunks : 0;
        w[u] = ok ? wpair[(size_t)b * KS + j] : 0.f;
        v[u] = o_part[((size_t)pos_of[(size_t)b * KS + j] * n_chunks + c) * d + i];
      }
#pragma unroll
      for (int u = 0; u < kCombItems; ++u) acc = fmaf(w[u], v[u], acc);
    }
  }
  part[sl][col] = acc;
  __syncthreads();
  if (sl == 0 && i < d) {
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < kCombSlices; ++k) s += part[k][col];
    Elem<T>::store(y + (size_t)b * d + i, s);
  }
}

}  // namespace

bool ffn_fused_supported(int d, int f, int max_count) {
  const int r = d / 256;
  return max_count <= 16 && d % 256 == 0 && (r == 1 || r == 2 || r == 4 || r == 8 || r == 16) && f % 32 == 0;
}

hipError_t launch_ffn_fused(hipStream_t s, const FfnArgs& a, KernelEvents ev) {
  if (a.g_max <= 0) return hipSuccess;
  dim3 grid(a.f / 32, a.g_max), block(64 * kFusedWaves);
  switch (a.d / 256) {
    case 1: launch_timed(ffn_fused_kernel<1>, grid, block, 0, s, ev, a); break;
    case 2: launch_timed(ffn_fused_kernel<2>, grid, block, 0, s, ev, a); break;
    case 4: launch_timed(ffn_fused_kernel<4>, grid, block, 0, s, ev, a); break;
    case 8: launch_timed(ffn_fused_kernel<8>, grid, block, 0, s, ev, a); break;
    case 16: launch_timed(ffn_fused_kernel<16>, grid, block, 0, s, ev, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_combine_chunks(hipStream_t s, const float* o_part, const float* wpair, const int32_t* pos_of,
                                 int B, int KS, int d, int n_chunks, void* y) {
  dim3 grid(B, (d + kCombCols - 1) / kCombCols), block(kCombCols * kCombSlices);
  hipLaunchKernelGGL(combine_chunks_kernel<uint16_t>, grid, block, 0, s, o_part, wpair, pos_of, KS, d, n_chunks,
                     (uint16_t*)y);
  return hipGetLastError();
}

}  // namespace moe
