// Expert SwiGLU FFN (paper section 2, Eq. 3) as a grouped bf16 GEMM for calls
// in which an expert sees many tokens (batched decode, prompt processing).
//
// One workgroup = 4 waves = a block of 64 output rows (4 MFMA row tiles, one
// per wave) of one expert x a tile of up to 128 of that expert's tokens.
//   * weights: A operand of v_mfma_f32_16x16x32_bf16, read by each wave straight
//     from global memory in the tiled layout (one coalesced KiB per fragment,
//     nontemporal: each fragment is used by exactly one wave of one token tile);
//   * tokens: B operand, shared by the four waves, staged through LDS in
//     fragment order (conflict-free 16-byte reads), double buffered two k-blocks
//     at a time so that the loads of stage s+1 overlap the MFMAs of stage s;
//   * accumulators: 8 column blocks x (gate, up) x 4 registers per lane.
// Column blocks beyond the expert's token count are skipped, so a large batch
// spread thinly over many experts degrades into weight streaming rather than
// wasted matrix work.  NMAT = 2 computes h = silu(X W_g^T) * (X W_u^T) (bf16,
// rows in group order); NMAT = 1 computes o = h W_d^T (fp32).
#include <type_traits>

#include "device_utils.hpp"
#include "moe_internal.hpp"

namespace moe {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));


// k-blocks (of 32) staged per step: two for the gate/up pass, one for the down projection (measured: the down pass
// has twice the workgroups over half the contraction length and runs 1.5x faster with the shorter stage)
template <int NMAT>
constexpr int kStageKbOf = NMAT == 2 ? 2 : 1;

// The 16 lanes that write the staged token tile together hold 16 / (4 kStageKb) consecutive token rows x all
// (k-block, 8-wide slice) combinations; without a swizzle those combinations fall on the same LDS banks.
// XOR-ing the row's position inside its 16-row block with this value spreads them over all banks; the reader
// applies the same value (measured: 4 % faster at 1024-2048 tokens per call).
template <int kStageKb>
__device__ __forceinline__ int swz(int q, int kbl) {
  return kStageKb == 4 ? q + 4 * kbl : kStageKb == 2 ? (q + 4 * kbl) * 2 : q * 4;
}

__device__ __forceinline__ const char* group_weights(const FfnArgs& a, int id) {
  return id < a.P ? a.buffers + (size_t)id * a.expert_bytes
                  : a.shared + (size_t)(id - a.P) * a.expert_bytes;
}

// kTokTile: tokens per workgroup (64, 128 or 256).  128 shares every weight fragment among more tokens; 64 needs half the
// accumulators and LDS, so more workgroups run side by side and hide each other's load latency: faster while an
// expert sees at most ~64 tokens (measured 169 against 212 us at 32 tokens per expert).
// (Holding more stages of weights in registers - three stages in flight instead of one - and fetching the tokens
// two stages ahead were both measured on the eight-wave variants at 128-1024 tokens per call: within +-3 %, and
// slower at 256; the one-stage look-ahead below stays.)
// kGemmWaves: row tiles (waves) per workgroup.  Eight waves share one staged token tile among 128 output rows,
// which halves the staging work per weight byte: faster once experts see ~128 tokens (302 against 335 us at 1024
// tokens per call, 488 against 576 us at 2048); four waves leave more workgroups per compute unit and are better
// below that.
// kSkb: k-blocks staged per step.  The default (two for gate/up, one for the down pass) suits launches with many
// workgroups per compute unit; a down pass with few workgroups and a long contraction (Mixtral-like: 512
// workgroups, 448 k-blocks) is bound by the latency of its one-KiB-per-wave steps and takes four k-blocks per step.
// kRing: stages of weight fragments a wave keeps in flight.  1: the next stage is requested while the current one
// multiplies (and the compiler waits for it at the end of the stage).  More: a ring with fixed slots, the stage loop
// unrolled kRing times, every load unconditional and the tokens requested ahead of the weights, so that waiting for
// the tokens of the next stage does not mean waiting for weights that are needed three stages later; the host
// picks it only when the number of stages is a multiple of kRing.
// kList: the (group, token tile) pairs come from the call's work list (gemm_worklist_kernel below) instead of the grid:
// blockIdx.y is an index into the list.
template <int NMAT, int kTokTile, int kGemmWaves, int kSkb = kStageKbOf<NMAT>, int kRing = 1, bool kList = false>
__global__ void __launch_bounds__(64 * kGemmWaves) ffn_gemm_kernel(FfnArgs a) {
  constexpr int kGemmThreads = 64 * kGemmWaves;
  constexpr int kColBlocks = kTokTile / 16;
  constexpr int kStageKb = kSkb;
  constexpr int kTotalPieces = kTokTile * kStageKb * 4;
  constexpr int kPieces = (kTotalPieces + kGemmThreads - 1) / kGemmThreads;
  constexpr bool kExact = kTotalPieces % kGemmThreads == 0;   // every thread stages kPieces pieces     // 16-byte pieces of the token tile each thread stages per step
  // [buffer][k-block in stage][column block][lane] x 16 bytes
  __shared__ u32x4 xs[2][kStageKb][kColBlocks][64];
  int tok0;
  GroupDesc gd;
  if constexpr (kList) {
    // the item carries what the workgroup needs of its group: one memory round trip instead of two before the
    // first weight request (the index is below the list's capacity, so the load needs no guard)
    const int32_t* list = a.t.pair_buf;
    const int n_items = list[NMAT == 2 ? 0 : 1];
    const int4 item = reinterpret_cast<const int4*>(list + 4)[(NMAT == 2 ? 0 : a.work_down) + blockIdx.y];
    if ((int)blockIdx.y >= n_items) return;
    tok0 = (item.x >> 16) * kTokTile;
    gd.buf = item.y; gd.begin = item.z; gd.count = item.w & 0x3fffffff; gd.miss = (item.w >> 30) & 1;
    gd.expert = -1; gd.pair0 = 0;
  } else {
    const int g = blockIdx.y;
    tok0 = blockIdx.z * kTokTile;
    const int ng = *a.t.n_groups;
    gd = a.t.grp[g];
    if (g >= ng) return;
  }
  if (a.pass != 2 && gd.miss != a.pass) return;
  const int cnt = gd.count;
  if (tok0 >= cnt) return;
  const int n_tok = min(kTokTile, cnt - tok0);       // tokens of this tile
  const int n_cb = (n_tok + 15) >> 4;                // column blocks in use

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int kdim = NMAT == 2 ? a.d : a.f;
  const int nkb = kdim >> 5;
  const int n_rt = (NMAT == 2 ? a.f : a.d) >> 4;
  const int rt = blockIdx.x * kGemmWaves + wave;     // this wave's row tile
  const bool has_rows = rt < n_rt;
  const int rtc = has_rows ? rt : n_rt - 1;          // clamped: loads stay in bounds, results are dropped

  // a group whose expert is not resident streams it from the pinned host pool (prompt streaming)
  const u32x4* w = (a.fetch != 0 && gd.miss != 0)
                       ? reinterpret_cast<const u32x4*>(a.pool + (size_t)gd.expert * a.expert_bytes)
                       : reinterpret_cast<const u32x4*>(group_weights(a, gd.buf));
  size_t kb_stride;
  if (NMAT == 2) {
    w += (size_t)rtc * nkb * 2 * 64 + lane;
    kb_stride = 2 * 64;
  } else {
    w += (size_t)2 * a.f * a.d / 8 + (size_t)rtc * 64 + lane;
    kb_stride = (size_t)(a.d >> 4) * 64;
  }

  // ring variant: the first weight stages are requested before the token addresses are looked up
  constexpr int kRingSlots = kRing > 1 ? kRing : 1;
  u32x4 wr[kRingSlots][kStageKb][NMAT];
  const int n_stages = nkb / kStageKb;            // ring variant: a multiple of kRing (host)
  auto req_w = [&](int slot, int s) {
    const int sc = s < n_stages ? s : n_stages - 1;
#pragma unroll
    for (int j = 0; j < kStageKb; ++j)
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
        wr[slot][j][m] = __builtin_nontemporal_load(w + (size_t)(sc * kStageKb + j) * kb_stride + m * 64);
  };
  if constexpr (kRing > 1) {
#pragma unroll
    for (int u = 0; u < kRing - 1; ++u) req_w(u, u);
  }

  // ---- staging assignment: 256 threads x kPieces pieces of 16 bytes = 128 rows x kStageKb k-blocks of 64 bytes ----
  const uint16_t* src[kPieces];
  int dst[kPieces];
#pragma unroll
  for (int i = 0; i < kPieces; ++i) {
    const int idx = threadIdx.x + kGemmThreads * i;
    const int r = idx / (4 * kStageKb), sg = idx % (4 * kStageKb);   // token row of the tile, 16-byte segment of it
    const int kbl = sg >> 2, q = sg & 3;
    dst[i] = (kExact || idx < kTotalPieces) ? (kbl * kColBlocks + (r >> 4)) * 64 + q * 16 + ((r & 15) ^ swz<kStageKb>(q, kbl)) : -1;
    if ((kExact || idx < kTotalPieces) && r < n_tok) {
      if (NMAT == 2) {
        const int p = a.t.sorted_pair[gd.begin + tok0 + r];
        src[i] = reinterpret_cast<const uint16_t*>(a.x) + (size_t)(p / a.KS) * a.d + sg * 8;
      } else {
        src[i] = reinterpret_cast<const uint16_t*>(a.h) + (size_t)(gd.begin + tok0 + r) * a.f + sg * 8;
      }
    } else {
      src[i] = nullptr;
    }
  }
  auto load_x = [&](u32x4 (&xr)[kPieces], int kb) {
#pragma unroll
    for (int i = 0; i < kPieces; ++i) {
      const int kbi = kb + ((threadIdx.x + kGemmThreads * i) % (4 * kStageKb)) / 4;   // k-block this piece belongs to
      xr[i] = (src[i] != nullptr && kbi < nkb) ? *reinterpret_cast<const u32x4*>(src[i] + (size_t)kb * 32)
                                                : u32x4{0, 0, 0, 0};
    }
  };
  auto load_w = [&](u32x4 (&wr)[kStageKb][NMAT], int kb) {
#pragma unroll
    for (int j = 0; j < kStageKb; ++j)
#pragma unroll
      for (int m = 0; m < NMAT; ++m)
        wr[j][m] = kb + j < nkb ? __builtin_nontemporal_load(w + (size_t)(kb + j) * kb_stride + m * 64)
                                : u32x4{0, 0, 0, 0};
  };

  f32x4 acc[kColBlocks][NMAT];
#pragma unroll
  for (int cb = 0; cb < kColBlocks; ++cb)
#pragma unroll
    for (int m = 0; m < NMAT; ++m) acc[cb][m] = f32x4{0.f, 0.f, 0.f, 0.f};

  if constexpr (kRing > 1) {
    constexpr int R = kRing;
    // pieces outside the tile read the first piece's address (always valid) and are zeroed on the way to LDS
    const uint16_t* srcv[kPieces];
    bool xok[kPieces];
#pragma unroll
    for (int i = 0; i < kPieces; ++i) {
      xok[i] = src[i] != nullptr;
      srcv[i] = xok[i] ? src[i] : reinterpret_cast<const uint16_t*>(NMAT == 2 ? a.x : a.h);
    }
    u32x4 xq[R][kPieces];
    auto req_x = [&](int slot, int s) {
      const int sc = s < n_stages ? s : n_stages - 1;
#pragma unroll
      for (int i = 0; i < kPieces; ++i)
        xq[slot][i] = *reinterpret_cast<const u32x4*>(srcv[i] + (size_t)sc * kStageKb * 32);
    };
    auto put_x = [&](int b, int slot) {
#pragma unroll
      for (int i = 0; i < kPieces; ++i)
        if (kExact || dst[i] >= 0) (&xs[b][0][0][0])[dst[i]] = xok[i] ? xq[slot][i] : u32x4{0, 0, 0, 0};
    };
    // tokens and weights of stage s are requested R - 1 stages before they are used
#pragma unroll
    for (int u = 0; u < R - 1; ++u) req_x(u, u);
    put_x(0, 0);
    __syncthreads();
    // the column blocks in use, rounded up to a quarter of the tile, as a compile-time count: no branch inside the
    // stage loop (column blocks beyond the tile's tokens hold zeros)
    auto run = [&](auto ncb_tag) {
      constexpr int NCB = decltype(ncb_tag)::value;
#pragma unroll 1
      for (int s0 = 0; s0 < n_stages; s0 += R) {
#pragma unroll
        for (int u = 0; u < R; ++u) {
          const int s = s0 + u;
          req_x((u + R - 1) % R, s + R - 1);  // tokens first: older than the weights requested next
          req_w((u + R - 1) % R, s + R - 1);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int j = 0; j < kStageKb; ++j) {
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
              const bf16x8 bfrag = __builtin_bit_cast(bf16x8, xs[u & 1][j][cb][lane ^ swz<kStageKb>(lane >> 4, j)]);
#pragma unroll
              for (int m = 0; m < NMAT; ++m)
                acc[cb][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wr[u][j][m]), bfrag,
                                                                     acc[cb][m], 0, 0, 0);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
          put_x((u & 1) ^ 1, (u + 1) % R);      // stage s + 1, requested two stages ago
          __syncthreads();
        }
      }
    };
    constexpr int Q = kColBlocks / 4;
    if (n_cb <= Q) run(std::integral_constant<int, Q>{});
    else if (n_cb <= 2 * Q) run(std::integral_constant<int, 2 * Q>{});
    else if (n_cb <= 3 * Q) run(std::integral_constant<int, 3 * Q>{});
    else run(std::integral_constant<int, kColBlocks>{});
  } else {
  u32x4 xr[kPieces], wc[kStageKb][NMAT], wn[kStageKb][NMAT];
  load_x(xr, 0);
  load_w(wc, 0);
#pragma unroll
  for (int i = 0; i < kPieces; ++i)
    if (kExact || dst[i] >= 0) (&xs[0][0][0][0])[dst[i]] = xr[i];
  __syncthreads();

  int buf = 0;
  for (int kb = 0; kb < nkb; kb += kStageKb) {
    const bool more = kb + kStageKb < nkb;
    if (more) {             // next stage's tokens and weights are fetched while this stage multiplies
      load_x(xr, kb + kStageKb);
      load_w(wn, kb + kStageKb);
    }
#pragma unroll
    for (int j = 0; j < kStageKb; ++j) {
#pragma unroll
      for (int cb = 0; cb < kColBlocks; ++cb) {
        if (cb < n_cb) {      // uniform
          const bf16x8 bfrag = __builtin_bit_cast(bf16x8, xs[buf][j][cb][lane ^ swz<kStageKb>(lane >> 4, j)]);
#pragma unroll
          for (int m = 0; m < NMAT; ++m)
            acc[cb][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wc[j][m]), bfrag,
                                                                 acc[cb][m], 0, 0, 0);
        }
      }
    }
    if (more) {
#pragma unroll
      for (int i = 0; i < kPieces; ++i)
        if (kExact || dst[i] >= 0) (&xs[buf ^ 1][0][0][0])[dst[i]] = xr[i];
#pragma unroll
      for (int j = 0; j < kStageKb; ++j)
#pragma unroll
        for (int m = 0; m < NMAT; ++m) wc[j][m] = wn[j][m];
    }
    __syncthreads();
    buf ^= 1;
  }
  }

  // ---- epilogue: lane holds rows (lane/16)*4 .. +3 of the row tile for token column lane%16 ----
  if (!has_rows) return;
  const int n = lane & 15, r4 = (lane >> 4) * 4;
#pragma unroll
  for (int cb = 0; cb < kColBlocks; ++cb) {
    const int tk = cb * 16 + n;
    if (cb < n_cb && tk < n_tok) {
      const size_t pos = (size_t)(gd.begin + tok0 + tk);
      if (NMAT == 2) {
        uint16_t hv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) hv[i] = f32_to_bf16(silu(acc[cb][0][i]) * acc[cb][NMAT - 1][i]);
        uint2 pk;
        pk.x = (uint32_t)hv[0] | ((uint32_t)hv[1] << 16);
        pk.y = (uint32_t)hv[2] | ((uint32_t)hv[3] << 16);
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.h) + pos * a.f + rt * 16 + r4) = pk;
      } else {
        *reinterpret_cast<f32x4*>(a.o + pos * a.d + rt * 16 + r4) = acc[cb][0];
      }
    }
  }
}

// The work list of a large call: one item per (group, token tile) that exists, groups with the most tokens first, for
// the gate/up pass (tiles of tile_up tokens) and for the down pass (tile_down).  Launching a grid of groups x the
// largest possible tile count instead leaves most workgroups empty (each still waits for its group record before it
// can tell), and the second and third tiles of the busy experts start last, a few dozen workgroups on an idle GPU
// (per-workgroup time stamps at 1024 tokens per call: 31 ms of workgroup time packed into 175 us on 256 units
// instead of 122).  The list lives in pair_buf, which nothing reads once the pairs are grouped:
// [0] items of the gate/up pass, [1] of the down pass, then 16-byte items from [4] on: gate/up items, and from item
// work_down on the down items; item = (group | tile << 16, buffer, begin, count | miss << 30): what a workgroup needs
// of its group record, so that it does not have to fetch that as well.  One workgroup of 256 threads, at most 256 groups.
__global__ void __launch_bounds__(256) gemm_worklist_kernel(CallTables t, int tile_up, int tile_down, int work_down) {
  __shared__ int s_cnt[256], s_first_up[256], s_first_down[256];
  const int ng = *t.n_groups;
  const int g = threadIdx.x;
  GroupDesc gd{};
  if (g < ng) gd = t.grp[g];
  const int cnt = gd.count;
  s_cnt[g] = cnt;
  __syncthreads();
  // position of the group when sorted by token count, largest first (ties by group index)
  int rank = 0;
  for (int j = 0; j < ng; ++j) rank += (s_cnt[j] > cnt || (s_cnt[j] == cnt && j < g)) ? 1 : 0;
  const int nu = (cnt + tile_up - 1) / tile_up, nd = (cnt + tile_down - 1) / tile_down;
  if (g < ng) { s_first_up[rank] = nu; s_first_down[rank] = nd; }
  __syncthreads();
  if (threadIdx.x == 0) {       // exclusive prefix sums in rank order (at most 256 short steps)
    int au = 0, ad = 0;
    for (int r = 0; r < ng; ++r) {
      const int u = s_first_up[r], d = s_first_down[r];
      s_first_up[r] = au; s_first_down[r] = ad;
      au += u; ad += d;
    }
    t.pair_buf[0] = au;
    t.pair_buf[1] = ad;
  }
  __syncthreads();
  if (g < ng) {
    int4* items = reinterpret_cast<int4*>(t.pair_buf + 4);
    const int w3 = cnt | ((gd.miss != 0 ? 1 : 0) << 30);
    for (int i = 0; i < nu; ++i) items[s_first_up[rank] + i] = int4{g | (i << 16), gd.buf, gd.begin, w3};
    for (int i = 0; i < nd; ++i) items[work_down + s_first_down[rank] + i] = int4{g | (i << 16), gd.buf, gd.begin, w3};
  }
}

}  // namespace

hipError_t launch_ffn_gemm(hipStream_t s, const FfnArgs& a, KernelEvents e1, KernelEvents e2) {
  if (a.g_max <= 0) return hipSuccess;
  // the group sizes are not known on the host; the mean load decides the token tile
  // (experts streamed from the host are read once per token tile: the large tile keeps that to one read up to 128 tokens)
  const int64_t load = (int64_t)a.max_count * a.KS;     // (token, expert) pairs of the call, all groups together
  constexpr int kSmallMax = 24;
  // (mean pairs per group; measured on the OLMoE-like layer: the 64-token tile on four waves is level with the
  // 128-token tile on eight waves up to ~24 and loses beyond - 165 against 147 us at 32, 243 against 205 us at 64 -
  // because the busier experts then need a second tile)
  const bool small_tile = a.fetch == 0 && load <= (int64_t)kSmallMax * a.g_max;
  // 256-token tiles: an expert with 129-256 tokens then streams its weights once instead of twice.  The gate/up
  // pass (both accumulator sets on the wave: 204 registers, one workgroup per compute unit) gains from a mean of ~52
  // pairs per expert on (118 against 126 us at 56, 164 against 184 us at 128; 113 against 103 us at 48); the down pass, which runs two workgroups per unit
  // with the 128-token tile, only from ~200 (180 against 188 us at 2048, but 126 against 109 us at 1024).
  constexpr int kBigUp = 52;
  const bool big_up = a.fetch == 0 && load > (int64_t)kBigUp * a.g_max;
  constexpr int kBigDown = 192;
  const bool big_down = a.fetch == 0 && load > (int64_t)kBigDown * a.g_max;
  const int waves = (small_tile || a.fetch != 0) ? 4 : 8;
  auto grid = [&](int rows, int tok_tile, int wv) {
    return dim3((rows / 16 + wv - 1) / wv, a.g_max, (a.max_count + tok_tile - 1) / tok_tile);
  };
  const dim3 b4(64 * 4), b8(64 * 8);
  // Large calls (measured on the OLMoE-like layer, gate/up + down: 188 against 200 us at 448 tokens per call, 193
  // against 210 at 512, 262 against 281 at 1024, 399 against 475 at 2048; level at 384, slower below): the ring
  // variant on 128-token tiles, its workgroups taken from a work list, for the gate/up pass from a mean of 40 pairs
  // per group, for the down pass from 56.
  constexpr int kRingUp = 40, kRingDown = 56, kRingTile = 128;
  const int cap = a.g_max + (int)(load / kRingTile);        // upper bound on the items of either list
  const bool listed = waves == 8 && a.g_max <= 256 && load >= (int64_t)kRingUp * a.g_max && 4 + 8 * cap <= load;
  const bool ring_up = listed && a.d % 256 == 0;                 // stages of two k-blocks, a multiple of four of them
  const bool ring_down = listed && load >= (int64_t)kRingDown * a.g_max && a.f % 128 == 0;
  FfnArgs b = a;
  b.work_down = cap;
  if (ring_up || ring_down)
    hipLaunchKernelGGL(gemm_worklist_kernel, dim3(1), dim3(256), 0, s, a.t, kRingTile, kRingTile, cap);
  // ---- gate/up ----
  if (small_tile) launch_timed(ffn_gemm_kernel<2, 64, 4>, grid(a.f, 64, 4), b4, 0, s, e1, a);
  else if (waves == 4) launch_timed(ffn_gemm_kernel<2, 128, 4>, grid(a.f, 128, 4), b4, 0, s, e1, a);
  else if (ring_up) launch_timed(ffn_gemm_kernel<2, kRingTile, 8, 2, 4, true>, dim3((a.f / 16 + 7) / 8, cap), b8, 0, s, e1, b);
  else if (big_up) launch_timed(ffn_gemm_kernel<2, 256, 8>, grid(a.f, 256, 8), b8, 0, s, e1, a);
  else launch_timed(ffn_gemm_kernel<2, 128, 8>, grid(a.f, 128, 8), b8, 0, s, e1, a);
  // ---- down ----
  // A long contraction with few output rows (Mixtral-like: d_ff = 14336, 8 experts) leaves the down pass with one
  // or two workgroups per compute unit, each waiting for one KiB per wave and step: four k-blocks per step and the
  // 64-row workgroups (measured on that layer: 205 against 314 us at 8 tokens per call).
  const bool deep_down = small_tile && a.f >= 4096 &&
                         (int64_t)((a.d / 16 + 3) / 4) * a.g_max < 4 * 256;
  if (deep_down) launch_timed(ffn_gemm_kernel<1, 64, 4, 4>, grid(a.d, 64, 4), b4, 0, s, e2, a);
  else if (small_tile) launch_timed(ffn_gemm_kernel<1, 64, 4>, grid(a.d, 64, 4), b4, 0, s, e2, a);
  else if (waves == 4) launch_timed(ffn_gemm_kernel<1, 128, 4>, grid(a.d, 128, 4), b4, 0, s, e2, a);
  else if (ring_down) launch_timed(ffn_gemm_kernel<1, kRingTile, 8, 1, 4, true>, dim3((a.d / 16 + 7) / 8, cap), b8, 0, s, e2, b);
  else if (big_down) launch_timed(ffn_gemm_kernel<1, 256, 8>, grid(a.d, 256, 8), b8, 0, s, e2, a);
  else launch_timed(ffn_gemm_kernel<1, 128, 8>, grid(a.d, 128, 8), b8, 0, s, e2, a);
  return hipGetLastError();
}

}  // namespace moe
