// Single-token decode call (paper section 2: router, Top-K, expert-cache lookups, SwiGLU experts of Eq. 3) on
// layers whose experts are too large for one workgroup per 32 intermediate rows to fit the GPU at once.
//
// The chunk kernel (ffn_fused.hip) launches d_ff / 32 workgroups per expert.  On a Mixtral-like layer that is
// 3.5 workgroups per compute unit: every one of them repeats the routing prologue, the last half round leaves
// compute units idle, and the combine reads 448 partial rows per expert.  Here the launch has ONE workgroup
// per compute unit: the 16-row tiles of an expert's intermediate dimension are dealt evenly (counts differ by
// at most one tile) to n_parts workgroups, n_parts * groups <= compute units.  A workgroup of eight waves
//   phase A: for each of its tiles, h[16 rows] = silu(W_g x) * (W_u x); the waves split the contraction
//            (k-block kb belongs to wave kb % 8), the partial tiles meet in LDS once, after the last tile;
//   phase B: o_part[d] = W_d[:, its rows] h: row tile rt of W_d belongs to wave rt % 8 and is accumulated over
//            the workgroup's k-blocks in one register tile; a k-block that straddles two workgroups is used half
//            by each (the lanes of the other half drop what they load and multiply zeros);
// and writes ONE partial row per (expert, workgroup): the combine reads n_parts rows per expert.
// Every wave runs one software-pipelined stream over all its fragments, D slots of 2 KiB in flight (a gate and an up
// fragment, or two W_d fragments), the first W_d loads under way while h is reduced.  The ring is a true rolling
// one: the loops are written so that the compiler waits for the oldest slot only (see the note at the loops), which
// is what lets a lone workgroup per compute unit keep the memory system busy; with the chunk kernel's loops
// (uniform branches around the loads: the ring drains where their paths meet) the DeepSeekMoE-like launch took
// 32.8 us, with these 30.5 us.  The launch is the whole call up to the combine: every workgroup runs the routing
// prologue of routed_prologue.hpp first (workgroups of shared experts skip it), one more row of the grid holds the
// bookkeeping workgroup.
#include <algorithm>

#include "device_utils.hpp"
#include "moe_internal.hpp"
#include "routed_prologue.hpp"

namespace moe {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTilesWaves = 8;
constexpr int kTilesMaxT = 16;      // tiles per workgroup the LDS scratch holds
constexpr int kXv = (kRoutedMaxX / 8 + 64 * kTilesWaves - 1) / (64 * kTilesWaves);

__device__ __forceinline__ u32x4 ldw(const u32x4* p) { return __builtin_nontemporal_load(p); }

// NPW = d / 256: k-blocks of the model dimension per wave and tile.
template <int NPW>
__global__ void __launch_bounds__(64 * kTilesWaves, 4) decode_tiles_kernel(FfnArgs a, RoutedArgs ra) {
  constexpr int WAVES = kTilesWaves;
  constexpr int D = NPW < 8 ? NPW : 8;     // ring depth: divides the per-tile and per-k-block item counts
  __shared__ float red[WAVES * 2 * 256];   // prologue scratch, then [tile][gate|up][wave][16 rows]
  __shared__ __align__(16) uint16_t hk[kTilesMaxT / 2 + 1][32];   // h of the workgroup's k-blocks, zero outside its rows
  __shared__ RoutedLds rl;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

  // A shared expert (group K and up of a one-token call) runs whatever the router says: its workgroups skip the
  // prologue and stream while the others still route - for that long the memory system is theirs alone.
  const int g = blockIdx.y;
  const bool always_on = g >= ra.a.K && g < a.g_max;
  GroupView gv;
  u32x4 xv[kXv];
  if (always_on) {
    gv.buf = a.P + (g - ra.a.K); gv.begin = g; gv.count = 1; gv.miss = 0; gv.expert = -1;
#pragma unroll
    for (int i = 0; i < kXv; ++i) {
      const int v = threadIdx.x + i * 64 * WAVES;
      xv[i] = v < a.d / 8 ? static_cast<const u32x4*>(a.x)[v] : u32x4{0, 0, 0, 0};
    }
  } else if (!routed_prologue<WAVES>(a, ra, rl, red, gv)) {
    return;
  }

  const int n = lane & 15, q = lane >> 4;
  const int d = a.d;
  const int nkb_d = d >> 5, n_dt = d >> 4;
  const int w = blockIdx.x, n_parts = a.n_parts;
  const int F16 = a.f >> 4;
  const int t0 = (int)((int64_t)w * F16 / n_parts), t1 = (int)((int64_t)(w + 1) * F16 / n_parts);
  const int T = t1 - t0;
  const int kb_lo = t0 >> 1, nkB = ((t1 - 1) >> 1) - kb_lo + 1;
  const bool lo_cut = (t0 & 1) != 0, hi_cut = (t1 & 1) != 0;   // first / last k-block shared with a neighbour

  const bool from_host = a.fetch != 0 && gv.miss != 0;
  const char* wdev = gv.buf < a.P ? a.buffers + (size_t)gv.buf * a.expert_bytes
                                  : a.shared + (size_t)(gv.buf - a.P) * a.expert_bytes;
  const char* wsrc = wdev;
  // Addresses are a wave-uniform byte pointer (scalar registers, advanced by scalar adds) plus a 32-bit lane offset.
  // gate/up fragment (tile, kb, m) sits at ((tile * nkb_d + kb) * 2 + m) KiB: item i of the wave = (tile t0 + i / NPW,
  // k-block wave + 8 (i % NPW)) is 16 KiB behind item i - 1.  W_d fragment (k-block, row tile) at (kb * n_dt + rt) KiB.
  const char* pa = wsrc + ((size_t)t0 * nkb_d + wave) * 2048;                              // next gate/up item to load
  const char* wb = wsrc + (size_t)2 * a.f * d * 2 + ((size_t)kb_lo * n_dt + wave) * 1024;  // W_d: (k-block kb_lo, row tile wave)
  const uint32_t lane_off = (uint32_t)lane * 16;
  // a lane whose half of a shared k-block is the neighbour's reads the address of the lane 32 away (the same cache
  // lines its own half needs anyway); the value is dropped when the fragment is used
  const uint32_t lane_off_cut = (uint32_t)(lane ^ 32) * 16;
  const bool low_half = q < 2;
  const int nbp = nkB * NPW;     // W_d fragments of a wave, in pairs: a ring slot holds 2 KiB in either phase
  float* orow = a.o + ((size_t)gv.begin * n_parts + w) * d;
  const uint16_t* xl = reinterpret_cast<const uint16_t*>(rl.xs) + (size_t)wave * 32 + q * 8;   // token 0, k-block `wave`
  auto at = [](const char* base, uint32_t off) { return reinterpret_cast<const u32x4*>(base + off); };

  // A group whose expert is not resident yet first copies its part of the expert from the pinned host pool (over
  // PCIe) into the group's device buffer, for this call and the calls to come, and then streams it like any other:
  // the copy takes 50 x as long as the streaming, and the loops below stay free of stores.
  if (from_host) {
    const char* src = a.pool + (size_t)gv.expert * a.expert_bytes;
    char* dst = const_cast<char*>(wdev);
    constexpr int U = 8, NT = 64 * WAVES;
    auto copy = [&](size_t first, size_t count, bool cut_aware) {      // in 16-byte units
      for (size_t c0 = threadIdx.x; c0 < count; c0 += (size_t)NT * U) {
        u32x4 v[U];
        bool take[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const size_t c = c0 + (size_t)u * NT;
          take[u] = c < count;
          if (cut_aware && take[u]) {      // halves of a shared k-block: the lanes' 512 bytes of every KiB
            const int kk = (int)(c / ((size_t)n_dt * 64));
            const bool low = (c & 63) < 32;
            take[u] = !((kk == 0 && lo_cut && low) || (kk == nkB - 1 && hi_cut && !low));
          }
          if (take[u]) v[u] = ldw(reinterpret_cast<const u32x4*>(src) + first + c);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (take[u]) reinterpret_cast<u32x4*>(dst)[first + c0 + (size_t)u * NT] = v[u];
      }
    };
    copy((size_t)t0 * nkb_d * 128, (size_t)T * nkb_d * 128, false);
    copy((size_t)2 * a.f * d / 8 + (size_t)kb_lo * n_dt * 64, (size_t)nkB * n_dt * 64, true);
    // the workgroup reads back what it wrote: stores out of the compute unit before anyone loads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
  }

  // Between the first load and the last use of the ring there is no branch with a global memory access inside
  // (results leave through LDS) and the scheduler may not move anything across the end of an item: the loads stay
  // one item apart and the compiler waits for exactly the oldest slot (s_waitcnt vmcnt(2 D - 2)) instead of
  // draining the ring.
  {
    u32x4 sg[D], su[D];
    // does this lane own its part of k-block kk of the workgroup?
    auto half_ok = [&](int kk) {
      return !((((kk == 0) & lo_cut) & low_half) | (((kk == nkB - 1) & hi_cut) & !low_half));
    };
    int kkI = 0;            // k-block (relative) of the W_d fragment the next load fetches
    const char* pb = wb;    // its row-tile base: row tile wave + 8 j
    auto load_b = [&]() {
      const uint32_t off = half_ok(kkI) ? lane_off : lane_off_cut;
      const u32x4 v = ldw(at(pb + (size_t)kkI * n_dt * 1024, off));
      const bool wrap = ++kkI == nkB;
      kkI = wrap ? 0 : kkI;
      pb += wrap ? 8 * 1024 : 0;
      return v;
    };
    auto issue_a = [&](int slot) {
      sg[slot] = ldw(at(pa, lane_off));
      su[slot] = ldw(at(pa, lane_off + 1024));
      pa += 16 * 1024;
    };
    auto issue_b = [&](int slot) {
      sg[slot] = load_b();
      su[slot] = load_b();
    };
#pragma unroll
    for (int u = 0; u < D; ++u) issue_a(u);       // T >= 2 tiles: at least 2 D gate/up items
    if (always_on) {        // the token reaches LDS behind the first weight loads
#pragma unroll
      for (int i = 0; i < kXv; ++i) {
        const int v = threadIdx.x + i * 64 * WAVES;
        if (v < a.d / 8) rl.xs[v] = xv[i];
      }
      __syncthreads();
    }

    // ---- phase A ----
    f32x4 accg, accu;
    auto a_step = [&](int u, const uint16_t* xg) {
      const bf16x8 xb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xg + (size_t)u * 256));
      accg = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, sg[u]), xb, accg, 0, 0, 0);
      accu = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, su[u]), xb, accu, 0, 0, 0);
    };
    auto a_done = [&](int t) {
      // every column of the B operand was token 0: the lanes of column 0 hold rows 4q .. 4q+3
      if (n == 0) {
        *reinterpret_cast<f32x4*>(&red[((t * 2 + 0) * WAVES + wave) * 16 + q * 4]) = accg;
        *reinterpret_cast<f32x4*>(&red[((t * 2 + 1) * WAVES + wave) * 16 + q * 4]) = accu;
      }
    };
    // the items of a tile come in R rounds of D (one per ring slot); all rounds but the very last load gate/up
    // items behind them, the last one hands its slots to phase B
    constexpr int R = NPW / D;
    accg = f32x4{0.f, 0.f, 0.f, 0.f}; accu = f32x4{0.f, 0.f, 0.f, 0.f};
    int t = 0, r = 0;
    for (int round = 0; round < T * R - 1; ++round) {
#pragma unroll
      for (int u = 0; u < D; ++u) {
        a_step(u, xl + (size_t)r * D * 256);
        issue_a(u);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (++r == R) {       // uniform; LDS only
        a_done(t);
        ++t;
        r = 0;
        accg = f32x4{0.f, 0.f, 0.f, 0.f}; accu = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
#pragma unroll
    for (int u = 0; u < D; ++u) {
      a_step(u, xl + (size_t)(R - 1) * D * 256);
      issue_b(u);
      __builtin_amdgcn_sched_barrier(0);
    }
    a_done(T - 1);
    __syncthreads();
    for (int i = threadIdx.x; i < nkB * 32; i += 64 * WAVES) {
      const int r16 = kb_lo * 32 + i;          // intermediate row
      const int tt = (r16 >> 4) - t0, row = r16 & 15;
      uint16_t hv = 0;
      if (tt >= 0 && tt < T) {
        float vg = 0.f, vu = 0.f;
#pragma unroll
        for (int k = 0; k < WAVES; ++k) {
          vg += red[((tt * 2 + 0) * WAVES + k) * 16 + row];
          vu += red[((tt * 2 + 1) * WAVES + k) * 16 + row];
        }
        hv = f32_to_bf16(silu(vg) * vu);
      }
      hk[i >> 5][i & 31] = hv;
    }
    __syncthreads();

    // ---- phase B: fragments in the order (row tile, k-block); a row tile is complete after nkB of them.  The
    //      running sum goes to LDS after every fragment (the last write of a row tile is the complete one) ----
    int kkC = 0;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float* ol = red + wave * 16 + q * 4;                  // [d] in LDS; the partial tiles of phase A are no longer needed
    auto consume_b = [&](u32x4 frag) {
      const bool ok = half_ok(kkC);
      frag = ok ? frag : u32x4{0, 0, 0, 0};
      const bf16x8 hb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(&hk[kkC][q * 8]));
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, frag), hb, acc, 0, 0, 0);
      if (n == 0) *reinterpret_cast<f32x4*>(ol) = acc;
      const bool wrap = ++kkC == nkB;      // uniform
      kkC = wrap ? 0 : kkC;
      ol += wrap ? WAVES * 16 : 0;
      acc = wrap ? f32x4{0.f, 0.f, 0.f, 0.f} : acc;
    };
    for (int p0 = 0; p0 < nbp - D; p0 += D) {
#pragma unroll
      for (int u = 0; u < D; ++u) {
        consume_b(sg[u]);
        consume_b(su[u]);
        issue_b(u);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int u = 0; u < D; ++u) {
      consume_b(sg[u]);
      consume_b(su[u]);
    }
  }
  __syncthreads();
  // the workgroup's partial row: coalesced, 16 bytes per thread
  for (int i = threadIdx.x; i < d / 4; i += 64 * WAVES)
    reinterpret_cast<f32x4*>(orow)[i] = reinterpret_cast<const f32x4*>(red)[i];
}

int npw_of(int d) {
  switch (d) {
    case 256: return 1;
    case 512: return 2;
    case 1024: return 4;
    case 2048: return 8;
    case 4096: return 16;
    default: return 0;
  }
}

}  // namespace

int decode_tiles_parts(int pool_layout, int d, int f, int batch, int groups, int n_cu, int E) {
  if (pool_layout != MOE_LAYOUT_TILED || batch != 1 || groups <= 0 || groups > n_cu) return 0;
  if (npw_of(d) == 0 || f % 32 != 0 || (E + 15) / 16 > 2 * kTilesWaves) return 0;
  const int chunks = f / 32;
  if (chunks * groups <= n_cu) return 0;      // the chunk kernel already has a compute unit per workgroup
  // Workgroups per group: at most one per compute unit in all, at least two tiles each.  Workgroups with one tile
  // more than the others finish alone, at the rate of a single compute unit, so the count within the upper quarter
  // of that range whose largest share is closest to the mean is taken (the smaller count on a tie), and the kernel
  // only if that share is within 10 % of the mean.  Measured per one-token call: Mixtral-like (896 tiles per
  // expert) 112 workgroups of 8 tiles 117.8 us, 128 of 7 119.7 us, chunk kernel 137 us; Phi-3.5-MoE-like (400
  // tiles) 100 workgroups of 4 tiles 59.7 us, 80 of 5 62.3 us, 128 of 3 or 4 67.4 us, chunk kernel 63.6 us;
  // DeepSeekMoE-like (88 tiles) 30 workgroups 32.7 us, 32: 33.1 us, 22 of 4 tiles 34.8 us, chunk kernel 39.8 us.
  const int n_max = std::min(chunks, n_cu / groups), f16 = f / 16;
  int n_parts = 0;
  int64_t best_num = 0;      // largest share * workgroups, to be compared as a fraction of f16
  for (int n = n_max; n >= 1 && 4 * n >= 3 * n_max; --n) {
    const int t_max = (f16 + n - 1) / n;
    if (t_max > kTilesMaxT) continue;
    const int64_t num = (int64_t)t_max * n;
    if (n_parts == 0 || num <= best_num) { n_parts = n; best_num = num; }
  }
  if (n_parts == 0 || best_num * 10 > (int64_t)f16 * 11) return 0;
  return n_parts;
}

hipError_t launch_decode_tiles(hipStream_t s, const FfnArgs& a, const RoutedArgs& ra, KernelEvents ev) {
  dim3 grid(a.n_parts, a.g_max + 1), block(64 * kTilesWaves);     // + the bookkeeping row
  switch (npw_of(a.d)) {
    case 1: launch_timed(decode_tiles_kernel<1>, grid, block, 0, s, ev, a, ra); break;
    case 2: launch_timed(decode_tiles_kernel<2>, grid, block, 0, s, ev, a, ra); break;
    case 4: launch_timed(decode_tiles_kernel<4>, grid, block, 0, s, ev, a, ra); break;
    case 8: launch_timed(decode_tiles_kernel<8>, grid, block, 0, s, ev, a, ra); break;
    case 16: launch_timed(decode_tiles_kernel<16>, grid, block, 0, s, ev, a, ra); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace moe
