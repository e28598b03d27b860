// Decode-shape expert FFN (paper section 2, Eq. 3) in ONE launch: gate/up
// projection, SiLU * up, and the down projection, for groups of at most 16
// tokens per expert, on bf16 experts in the tiled layout (the host uses it for calls of up to 6 tokens; the grouped
// GEMM is faster beyond).
//
// Why one launch: at decode an expert sees one or a few tokens, every weight
// byte is used once, and a whole layer call moves only ~100 MB - about 13 us of
// HBM time.  Two dependent kernels pay the launch ramp, the metadata round trip
// and the drain twice; here they are paid once.
//
// A workgroup owns one expert and one chunk of 32 rows of its intermediate
// dimension (one MFMA k-block of the down projection):
//   phase A: h[32 rows] = silu(W_g[rows,:] x) * (W_u[rows,:] x).  The waves are
//     2 row tiles x (waves/2) slices of the contraction; partial tiles meet in LDS.
//   phase B: partial o[:, d] = W_d[:, rows] h[rows]; the row tiles of W_d are
//     dealt round-robin to the waves; with the chunk as the only k-block every MFMA result is a
//     finished partial sum, written as [pair][chunk][d] fp32.
// The chunks of an expert are summed, in chunk order, by combine_chunks_kernel
// together with the gate-weighted sum over experts of Eq. 2 (deterministic).
//
// Each wave runs ONE software-pipelined stream over its fragments - first its
// gate/up fragments (with the matching token slices), then its W_d fragments -
// with up to kDepth fragments in flight; the W_d loads are already under way
// while the workgroup reduces h, so HBM never idles inside the workgroup.
#include <algorithm>
#include <type_traits>

#include "device_utils.hpp"
#include "moe_internal.hpp"
#include "routed_prologue.hpp"

namespace moe {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// waves per workgroup = 2 row tiles x (waves/2) contraction slices; chosen per launch from the grid size
constexpr int kDepth = 8;     // fragments (gate+up pairs count as one) a wave keeps in flight

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Weight fragments are read exactly once per call: nontemporal loads keep them from
// displacing the router matrix, the tokens and the partial sums from L2 / Infinity Cache
// (measured: +8 % on the 700 MB Mixtral-like call, and the router kernel of the next
// call finds its matrix still cached).
__device__ __forceinline__ u32x4 ldw(const u32x4* p) { return __builtin_nontemporal_load(p); }

__device__ __forceinline__ const char* group_weights(const FfnArgs& a, int id) {
  return id < a.P ? a.buffers + (size_t)id * a.expert_bytes
                  : a.shared + (size_t)(id - a.P) * a.expert_bytes;
}

// One layer's router matrix [E][d] (row-major) -> [ceil(E/16)][d/32][64 lanes][8]: lane l, element j of fragment
// (tile, kb) = W_r[16 tile + l % 16][32 kb + 8 (l / 16) + j]; rows beyond E are zero.
__global__ void pack_router_kernel(const uint16_t* __restrict__ w, uint16_t* __restrict__ out, int E, int d, int n_layers) {
  const int nkb = d >> 5, tiles = (E + 15) >> 4;
  const size_t per_layer = (size_t)tiles * nkb * 512;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= per_layer * n_layers) return;
  const size_t l = i / per_layer, r = i - l * per_layer;
  const int j = (int)(r & 7), lane = (int)((r >> 3) & 63);
  const size_t frag = r >> 9;
  const int kb = (int)(frag % nkb), tile = (int)(frag / nkb);
  const int e = tile * 16 + (lane & 15);
  out[i] = e < E ? w[(l * E + e) * d + (size_t)kb * 32 + (lane >> 4) * 8 + j] : (uint16_t)0;
}

// SLOT0 = (gate/up items per wave) % kDepth: the ring slot in which the first W_d fragment of a wave sits.
// ROUTED: the launch is the decode call up to the combine.  Every workgroup first derives the routing, the cache
// lookups and the groups for itself (prologue above), then runs its chunk.  (Reducing the partial sums in the same
// launch was built and measured: the workgroups have to meet at a device-scope counter, and on this GPU that
// meeting alone - 8 us for 256 workgroups, far more with release/acquire fences, which write back and invalidate
// whole L2 caches - costs more than the separate combine launch.)
template <int WAVES, int SLOT0, bool ROUTED>
__device__ __forceinline__ void fused_body(const FfnArgs& a, const RoutedArgs* rap) {
  __shared__ float red[WAVES][2][256];            // partial gate / up tiles of the waves
  __shared__ __align__(16) uint16_t hs[16][32];   // h of the chunk, bf16, [token][row in chunk]
  __shared__ typename std::conditional<ROUTED, RoutedLds, int>::type rl_store;
  const int g = blockIdx.y;
  const int lane = threadIdx.x & 63;
  // (the wave index is the same in all lanes of a wave: saying so keeps everything derived from it - row tile,
  // contraction slice, fragment offsets - in scalar registers)
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = blockIdx.x;  // chunk of 32 intermediate rows

  int gd_buf, gd_begin, gd_count, gd_miss, gd_expert, gd_pair0;
  if constexpr (ROUTED) {
    GroupView gv;
    if (!routed_prologue<WAVES>(a, *rap, rl_store, &red[0][0][0], gv)) return;
    gd_buf = gv.buf; gd_begin = gv.begin; gd_count = gv.count; gd_miss = gv.miss; gd_expert = gv.expert;
    gd_pair0 = 0;
  } else {
    const int ng = *a.t.n_groups;        // both loads are issued before the first branch: one round trip
    const GroupDesc gd = a.t.grp[g];
    if (g >= ng || (a.pass != 2 && gd.miss != a.pass)) return;
    gd_buf = gd.buf; gd_begin = gd.begin; gd_count = gd.count; gd_miss = gd.miss; gd_expert = gd.expert;
    gd_pair0 = gd.pair0;
  }

  const int n = lane & 15;   // token column
  const int q = lane >> 4;   // 8-wide slice of a 32-deep k-block
  const int d = a.d;
  const int nkb_d = d >> 5, n_dt = d >> 4;
  constexpr int KS = WAVES / 2;
  const int tile = wave & 1, ks = wave >> 1;
  const int na = nkb_d / KS;      // gate/up k-blocks of this wave   (host guarantees divisibility)
  const int nb = n_dt / WAVES;    // W_d row tiles of this wave
  // k-blocks are dealt round-robin to the contraction slices, so the waves of a row tile read
  // adjacent KiBs at any moment (measured 4 % faster than one contiguous run per wave)
  const int kb0 = ks, kb_step = KS;

  const size_t x_step = (size_t)kb_step * 32, w_step = (size_t)kb_step * 128;
  // a group whose expert is not resident yet reads it from the pinned host pool over PCIe and, on the way,
  // fills its device buffer for the calls to come (fetch fused into the compute: no copy engine, no host)
  const bool from_host = a.fetch != 0 && gd_miss != 0;
  const char* wdev = group_weights(a, gd_buf);
  const char* wsrc = from_host ? a.pool + (size_t)gd_expert * a.expert_bytes : wdev;
  const intptr_t fill_delta = reinterpret_cast<intptr_t>(wdev) - reinterpret_cast<intptr_t>(wsrc);
  const u32x4* wbase = reinterpret_cast<const u32x4*>(wsrc);
  auto fill = [&](const u32x4* src, u32x4 v) {     // same offset inside the device block
    *reinterpret_cast<u32x4*>(reinterpret_cast<intptr_t>(src) + fill_delta) = v;
  };
  // gate/up fragment (row tile 2c+tile, kb, m) and W_d fragment (chunk c, row tile dt)
  const u32x4* wa = wbase + ((size_t)(2 * c + tile) * nkb_d + kb0) * 2 * 64 + lane;
  const u32x4* wb = wbase + (size_t)2 * a.f * d / 8 + ((size_t)c * n_dt + wave) * 64 + lane;

  const int begin = gd_begin, cnt = gd_count;
  const uint16_t* xrow = nullptr;
  if (n < cnt) {
    int p;
    if constexpr (ROUTED) p = rl_store.sorted_pair[begin + n];
    else p = n == 0 ? gd_pair0 : a.t.sorted_pair[begin + n];   // a single-token group needs no second look-up
    xrow = reinterpret_cast<const uint16_t*>(a.x) + (size_t)(p / a.KS) * d + (size_t)kb0 * 32 + q * 8;
  }

  // ---- one pipelined stream per wave: na gate/up items, then nb W_d items, kDepth in flight ----
  // ring slot u holds item (base + u); an item is issued into the slot of the item consumed kDepth earlier
  u32x4 sg[kDepth], su[kDepth], sx[kDepth];
  const int total = na + nb;
  auto issue = [&](int slot, int item) {
    if (item < na) {
      sx[slot] = xrow ? *reinterpret_cast<const u32x4*>(xrow + (size_t)item * x_step) : u32x4{0, 0, 0, 0};
      sg[slot] = ldw(wa + (size_t)item * w_step);
      su[slot] = ldw(wa + (size_t)item * w_step + 64);
    } else if (item < total) {
      sg[slot] = ldw(wb + (size_t)(item - na) * WAVES * 64);
    }
  };
#pragma unroll
  for (int u = 0; u < kDepth; ++u) issue(u, u);

  f32x4 accg = {0.f, 0.f, 0.f, 0.f}, accu = {0.f, 0.f, 0.f, 0.f};
  for (int base = 0; base < na; base += kDepth) {
#pragma unroll
    for (int u = 0; u < kDepth; ++u) {
      if (base + u < na) {      // uniform
        const bf16x8 xb = __builtin_bit_cast(bf16x8, sx[u]);
        accg = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, sg[u]), xb, accg, 0, 0, 0);
        accu = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, su[u]), xb, accu, 0, 0, 0);
        if (from_host) {
          fill(wa + (size_t)(base + u) * w_step, sg[u]);
          fill(wa + (size_t)(base + u) * w_step + 64, su[u]);
        }
        issue(u, base + u + kDepth);
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
    const int src = ((mm >> 2) * 16 + nn) * 4 + (mm & 3);       // where the MFMA left element (mm, nn)
    float vg = 0.f, vu = 0.f;
#pragma unroll
    for (int k = 0; k < KS; ++k) {
      vg += red[k * 2 + tl][0][src];
      vu += red[k * 2 + tl][1][src];
    }
    hs[nn][tl * 16 + mm] = nn < cnt ? f32_to_bf16(silu(vg) * vu) : (uint16_t)0;
  }
  __syncthreads();

  // ---- phase B: W_d[:, chunk] h; the first W_d fragments are already in their ring slots ----
  const bf16x8 hb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(&hs[n][q * 8]));
  const size_t n_chunks = (size_t)(a.f >> 5);
  float* obase = a.o + ((size_t)(begin + n) * n_chunks + c) * d + (lane >> 4) * 4;
  // item (na + j) sits in ring slot (na + j) % kDepth: the slot sequence continues where phase A stopped
  for (int base = 0; base < nb; base += kDepth) {
#pragma unroll
    for (int u = 0; u < kDepth; ++u) {
      const int j = base + u;
      if (j < nb) {             // uniform
        const int v = (SLOT0 + u) % kDepth;   // compile-time after unrolling
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, sg[v]), hb, acc, 0, 0, 0);
        if (from_host) fill(wb + (size_t)j * WAVES * 64, sg[v]);
        issue(v, na + j + kDepth);
        // lane holds rows (lane/16)*4 .. +3 of row tile (wave + WAVES j) for token n
        if (n < cnt)
          *reinterpret_cast<f32x4*>(obase + (size_t)(wave + WAVES * j) * 16) = acc;
      }
    }
  }

}

template <int WAVES, int SLOT0>
__global__ void __launch_bounds__(64 * WAVES) ffn_fused_kernel(FfnArgs a) {
  fused_body<WAVES, SLOT0, false>(a, nullptr);
}

// (second launch bound: four waves per SIMD, i.e. at most 128 registers, so that as many workgroups are
// resident at once as with the plain expert kernel)
template <int WAVES, int SLOT0>
__global__ void __launch_bounds__(64 * WAVES, 4) decode_single_kernel(FfnArgs a, RoutedArgs ra) {
  fused_body<WAVES, SLOT0, true>(a, &ra);
}

// y[b][i] = sum_j wpair[b][j] * sum_c o_part[pos_of[b][j]][c][i].
// A workgroup owns 32 columns (128 bytes of every partial row) of one token: 8 lanes x 4 columns, 128 slices.
// The slices split the KS * n_chunks partial rows; a thread reads 16 bytes per row, all loads of a batch issued
// before the first use.  The slices are then summed in a fixed order (butterfly inside the wave, wave order in
// LDS), so the result does not depend on timing.
constexpr int kCombLanes = 8, kCombSlices = 128, kCombBatch = 8;

// IDENT: pair (b, j) sits at partial row b * KS + j (a call of one token through the single-launch decode keeps its
// pairs in order), so the addresses of the partial rows do not wait for pos_of: one memory round trip instead of two.
template <typename T, bool IDENT>
__global__ void __launch_bounds__(kCombLanes * kCombSlices)
combine_chunks_kernel(const float* __restrict__ o_part, const float* __restrict__ wpair,
                      const int32_t* __restrict__ pos_of, int KS, int d, int n_chunks, T* __restrict__ y) {
  __shared__ f32x4 part[kCombSlices / 8][kCombLanes];
  const int b = blockIdx.x;
  const int cl = threadIdx.x % kCombLanes, sl = threadIdx.x / kCombLanes;
  const int col = blockIdx.y * (kCombLanes * 4) + cl * 4;       // host guarantees d % 32 == 0
  const int n_items = KS * n_chunks;
  const int per = (n_items + kCombSlices - 1) / kCombSlices;
  const int it_end = min((sl + 1) * per, n_items);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int it0 = sl * per; it0 < it_end; it0 += kCombBatch) {
    f32x4 v[kCombBatch];
    float w[kCombBatch];
#pragma unroll
    for (int u = 0; u < kCombBatch; ++u) {
      const int it = it0 + u;
      const bool ok = it < it_end;
      const int j = ok ? it / n_chunks : 0, c = ok ? it - j * n_chunks : 0;
      w[u] = ok ? wpair[(size_t)b * KS + j] : 0.f;
      const size_t row = IDENT ? (size_t)b * KS + j : (size_t)pos_of[(size_t)b * KS + j];
      v[u] = *reinterpret_cast<const f32x4*>(o_part + (row * n_chunks + c) * d + col);
    }
#pragma unroll
    for (int u = 0; u < kCombBatch; ++u) acc += w[u] * v[u];
  }
  // the 8 slices of a wave (lane bits 3..5), then the 16 waves
#pragma unroll
  for (int m = 8; m < 64; m <<= 1) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] += __shfl_xor(acc[i], m);
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (lane < kCombLanes) part[wave][lane] = acc;
  __syncthreads();
  if (threadIdx.x < kCombLanes) {
    f32x4 sum = part[0][threadIdx.x];
#pragma unroll
    for (int k = 1; k < kCombSlices / 8; ++k) sum += part[k][threadIdx.x];
#pragma unroll
    for (int i = 0; i < 4; ++i) Elem<T>::store(y + (size_t)b * d + col + i, sum[i]);
  }
}

}  // namespace

namespace {

// 2 x (waves/2) phase-A split and waves-way phase-B split must divide evenly; the ring hand-over between the
// phases needs the per-wave gate/up count to be a multiple of the ring depth, or one of the small counts compiled
bool waves_ok(int d, int waves) {
  if (d % (16 * waves) != 0) return false;
  const int na = (d / 32) / (waves / 2);
  return na % kDepth == 0 || na == 1 || na == 2 || na == 4;
}

// Small grids need many waves per workgroup to have enough loads in flight; large grids stream best with small
// workgroups (less time lost at the workgroup barriers).  Measured on MI355X.
int pick_waves(int d, int n_workgroups) {
  const int pref = n_workgroups <= 256 ? 8 : 4;     // eight waves only while every workgroup has a compute unit to itself
  for (int w : {pref, 8, 4, 16})
    if (waves_ok(d, w)) return w;
  return 0;
}

template <int WAVES>
void launch_fused_waves(hipStream_t s, const FfnArgs& a, KernelEvents ev) {
  dim3 grid(a.f / 32, a.g_max), block(64 * WAVES);
  const int na = (a.d / 32) / (WAVES / 2);
  switch (na % kDepth) {
    case 0: launch_timed(ffn_fused_kernel<WAVES, 0>, grid, block, 0, s, ev, a); break;
    case 1: launch_timed(ffn_fused_kernel<WAVES, 1>, grid, block, 0, s, ev, a); break;
    case 2: launch_timed(ffn_fused_kernel<WAVES, 2>, grid, block, 0, s, ev, a); break;
    default: launch_timed(ffn_fused_kernel<WAVES, 4>, grid, block, 0, s, ev, a); break;
  }
}

template <int WAVES>
void launch_single_waves(hipStream_t s, const FfnArgs& a, const RoutedArgs& ra, KernelEvents ev) {
  dim3 grid(a.f / 32, a.g_max + 1), block(64 * WAVES);     // + the bookkeeping row
  const int na = (a.d / 32) / (WAVES / 2);
  switch (na % kDepth) {
    case 0: launch_timed(decode_single_kernel<WAVES, 0>, grid, block, 0, s, ev, a, ra); break;
    case 1: launch_timed(decode_single_kernel<WAVES, 1>, grid, block, 0, s, ev, a, ra); break;
    case 2: launch_timed(decode_single_kernel<WAVES, 2>, grid, block, 0, s, ev, a, ra); break;
    default: launch_timed(decode_single_kernel<WAVES, 4>, grid, block, 0, s, ev, a, ra); break;
  }
}

}  // namespace

size_t router_packed_bytes(int E, int d) { return (size_t)((E + 15) / 16) * (size_t)(d / 32) * 1024; }

hipError_t launch_pack_router(hipStream_t s, const void* router_w, void* out, int E, int d, int n_layers) {
  const size_t n = router_packed_bytes(E, d) / 2 * (size_t)n_layers;
  hipLaunchKernelGGL(pack_router_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                     static_cast<const uint16_t*>(router_w), static_cast<uint16_t*>(out), E, d, n_layers);
  return hipGetLastError();
}

bool decode_single_supported(int pool_layout, int policy, int E, int C, int P, int n_shared, int K, int d, int f,
                             int batch) {
  if (!fast_table(policy, C, P, n_shared)) return false;
  if (batch > kRoutedMaxB || batch * d > kRoutedMaxX || batch * (K + n_shared) > kWave || E > kRoutedMaxE) return false;
  int waves = 0;
  if (pool_layout == MOE_LAYOUT_TILED_INT4) {
    if (!ffn_fused_q4_supported(d, f, batch)) return false;
    waves = fused_q4_waves(d);
  } else if (pool_layout == MOE_LAYOUT_TILED) {
    if (!ffn_fused_supported(d, f, batch)) return false;
    const int g_max = std::min(batch * K, P) + n_shared;
    waves = pick_waves(d, (f / 32) * g_max);
  }
  return waves != 0 && (E + 15) / 16 <= 2 * waves;      // the logit tiles of the waves fit their LDS scratch
}

hipError_t launch_decode_single(hipStream_t s, int pool_layout, const FfnArgs& a, const RoutedArgs& ra, KernelEvents ev) {
  if (pool_layout == MOE_LAYOUT_TILED_INT4) return launch_decode_single_q4(s, a, ra, ev);
  switch (pick_waves(a.d, (a.f / 32) * a.g_max)) {
    case 4: launch_single_waves<4>(s, a, ra, ev); break;
    case 8: launch_single_waves<8>(s, a, ra, ev); break;
    case 16: launch_single_waves<16>(s, a, ra, ev); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

bool ffn_fused_supported(int d, int f, int max_count) {
  return max_count <= fused_max_tokens(f) && f % 32 == 0 && pick_waves(d, 1) != 0;
}

hipError_t launch_ffn_fused(hipStream_t s, const FfnArgs& a, KernelEvents ev) {
  if (a.g_max <= 0) return hipSuccess;
  // the grid is sized by an upper bound on the groups; batch 1 fills it exactly
  switch (pick_waves(a.d, (a.f / 32) * a.g_max)) {
    case 4: launch_fused_waves<4>(s, a, ev); break;
    case 8: launch_fused_waves<8>(s, a, ev); break;
    case 16: launch_fused_waves<16>(s, a, ev); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_combine_chunks(hipStream_t s, const float* o_part, const float* wpair, const int32_t* pos_of,
                                 int B, int KS, int d, int n_chunks, void* y, bool identity) {
  dim3 grid(B, d / (kCombLanes * 4)), block(kCombLanes * kCombSlices);
  if (identity)
    hipLaunchKernelGGL((combine_chunks_kernel<uint16_t, true>), grid, block, 0, s, o_part, wpair, pos_of, KS, d,
                       n_chunks, (uint16_t*)y);
  else
    hipLaunchKernelGGL((combine_chunks_kernel<uint16_t, false>), grid, block, 0, s, o_part, wpair, pos_of, KS, d,
                       n_chunks, (uint16_t*)y);
  return hipGetLastError();
}

}  // namespace moe
