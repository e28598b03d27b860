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
#include "gating.hpp"
#include "moe_internal.hpp"

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

// ---------------------------------------------------------------- single-launch decode: prologue pieces
// Limits of the routed variant: tokens per call, experts whose logits a workgroup keeps, token elements staged.
constexpr int kRoutedMaxB = 4, kRoutedMaxE = 256, kRoutedMaxX = 8192;

// What every workgroup of the routed variant derives for itself, in LDS.
struct RoutedLds {
  u32x4 xs[kRoutedMaxX / 8];            // the call's tokens [B][d], bf16
  float zs[kRoutedMaxB][kRoutedMaxE];   // router logits of the call's tokens
  float bias[kRoutedMaxB * kRoutedMaxE];// the call's logit bias (zeros when there is none)
  int32_t buf_of[kRoutedMaxE];          // expert -> buffer that holds it before the call, -1 if not resident
  int32_t idx[64];                      // [B][K] selected experts, ascending id
  float wpair[64];                      // [B][KS] gate weights (1 for shared experts); bookkeeping workgroup only
  int32_t sorted_pair[64], pos_of[64];  // pairs ordered by group, and the inverse
  int32_t g_buf[64], g_begin[64], g_count[64], g_miss[64], g_expert[64];   // groups
  int32_t n_groups, status;
};

// Cache lookups and grouping of a call of at most 64 (token, expert) pairs on the register-resident LRU table
// (section 2, "Expert Offloading Systems"; lazy LRU = the gamma -> 0+ member of Definition C.1).  Runs in ONE
// wave of EVERY workgroup on the same inputs, so all of them reach the same groups; only the bookkeeping
// workgroup (`commit`) writes the table after the call (to st_out), the trace, the counters and the call record.
// A workgroup that does not commit and finds every selected expert in the map expert -> buffer (rl.buf_of) skips the
// lookups: it needs the buffers, not the recency updates.
__device__ void lookup_small(FastTable f, RoutedLds& rl, const RoutedArgs& ra, const CallTables& t, bool commit) {
  const CacheCallArgs& a = ra.a;
  const int lane = threadIdx.x & 63;
  const int C = a.C, P = a.P, K = a.K, KS = a.KS;
  const FastTable f0 = f;       // as loaded: written back unchanged should the call fail
  {   // buffers released by the previous call: all its kernels have finished, reuse them
    const int src = lane - f.n_free;
    const int z = __shfl(f.zomb, src < 0 ? 0 : src);
    if (src >= 0 && src < f.n_zombie) f.free_b = z;
    f.n_free += f.n_zombie;
    f.n_zombie = 0;
  }
  const uint32_t seq = a.seq;
  const int n_lookups = a.B * K, NP = a.B * KS;
  int status = MOE_OK, n_miss = 0, n_evict = 0, n_hits = 0;
  const int my_e = lane < n_lookups ? rl.idx[lane] : -3;
  int my_buf = -1, my_hit = 0, my_evicted = -1;     // lane q: outcome of lookup q
  int filled = 0;                                    // lane p: expert + 1 this call brings into buffer p

  // ---- the resident regime first: when every lookup hits, residency does not change and the recency updates
  //      commute (the last lookup of a slot decides its tick); nothing is changed unless all of them hit ----
  bool all_hit = f.n_res > 0;
  bool resolved = false;
  if (!commit) {
    const int pre = lane < n_lookups ? rl.buf_of[my_e] : 0;
    if (__ballot(pre < 0) == 0) { my_buf = pre; resolved = true; }
  }
  if (!resolved) {
    int my_slot = 0;
    uint64_t new_tick = f.tick;
    for (int q = 0; q < n_lookups && all_hit; ++q) {       // uniform
      const uint64_t hm = __ballot(f.exp == readlane_i(my_e, q));
      if (hm == 0) { all_hit = false; break; }
      const int s = __ffsll((unsigned long long)hm) - 1;
      if (lane == q) my_slot = s;
      if (lane == s) new_tick = (uint64_t)(f.clock + q + 1);
    }
    if (all_hit) {
      f.tick = new_tick;
      my_buf = __shfl(f.buf, my_slot);                // lane q: buffer that lookup q reads
      for (int q = 0; q < n_lookups; ++q)
        if (lane == readlane_i(my_buf, q)) f.used = seq;
      my_hit = 1;
      f.clock += n_lookups;
      n_hits = n_lookups;
    }
  }
  for (int q = 0; q < n_lookups && !all_hit && !resolved; ++q) {  // in order: each lookup changes what the next one sees
    const int e = readlane_i(my_e, q);
    const uint64_t hm = __ballot(f.exp == e);
    int s, buf, evicted = -1;
    const bool hit = hm != 0;
    if (hit) {
      s = __ffsll((unsigned long long)hm) - 1;
      buf = readlane_i(f.buf, s);
      ++n_hits;
    } else {
      if (f.n_res < C) {          // slots fill in index order, so the lowest empty slot is n_res
        s = f.n_res++;
        buf = readlane_i(f.free_b, --f.n_free);
      } else {
        s = wave_argmin_tick(f.tick);
        evicted = readlane_i(f.exp, s);
        const int vb = readlane_i(f.buf, s);
        if ((uint32_t)readlane_i((int)f.used, vb) == seq) {   // an earlier token of this call reads it
          if (f.n_free == 0) { status = MOE_ERR_STAGING_EXHAUSTED; break; }
          buf = readlane_i(f.free_b, --f.n_free);
          if (lane == f.n_zombie) f.zomb = vb;
          ++f.n_zombie;
        } else {
          buf = vb;
        }
        ++n_evict;
      }
      if (lane == s) { f.exp = e; f.buf = buf; }
      if (lane == buf) filled = e + 1;
      ++n_miss;
    }
    ++f.clock;
    if (lane == s) f.tick = (uint64_t)f.clock;
    if (lane == buf) f.used = seq;
    if (lane == q) { my_buf = buf; my_hit = hit ? 1 : 0; my_evicted = evicted; }
  }

  // ---- groups: the pairs that read the same buffer ----
  int n_groups = 0, rank = 0;
  if (status == MOE_OK) {
    const int b = lane / KS, k = lane - b * KS;
    int my_pair = __shfl(my_buf, k < K ? b * K + k : 0);
    if (lane >= NP) my_pair = -1;
    else if (k >= K) my_pair = P + (k - K);       // shared experts
    const int was_filled = __shfl(filled, my_pair < P && my_pair >= 0 ? my_pair : 0);
    const int fe = my_pair < P ? was_filled : 0;
    if (a.B == 1) {
      // one token: its experts are distinct, every pair is its own group, in the order of the pairs
      rank = lane;
      if (lane < NP) {
        rl.sorted_pair[lane] = lane; rl.pos_of[lane] = lane;
        rl.g_buf[lane] = my_pair; rl.g_begin[lane] = lane; rl.g_count[lane] = 1;
        rl.g_miss[lane] = fe != 0; rl.g_expert[lane] = fe - 1;
      }
      n_groups = NP;
    } else {
      // lane p = b*KS + k ranks its pair against all others (stable); groups in ascending buffer id
      int same_before = 0, cnt = 0;
      for (int q = 0; q < NP; ++q) {
        const int bq = readlane_i(my_pair, q);
        rank += (bq < my_pair || (bq == my_pair && q < lane)) ? 1 : 0;
        cnt += bq == my_pair ? 1 : 0;
        same_before += (bq == my_pair && q < lane) ? 1 : 0;
      }
      const bool is_first = lane < NP && same_before == 0;
      const uint64_t fm = __ballot(is_first);
      int gidx = 0;
      for (uint64_t m = fm; m != 0; m &= m - 1) {
        const int q = __ffsll((unsigned long long)m) - 1;
        gidx += readlane_i(my_pair, q) < my_pair ? 1 : 0;
      }
      if (lane < NP) {
        rl.sorted_pair[rank] = lane;
        rl.pos_of[lane] = rank;
        if (is_first) {
          rl.g_buf[gidx] = my_pair; rl.g_begin[gidx] = rank; rl.g_count[gidx] = cnt;
          rl.g_miss[gidx] = fe != 0; rl.g_expert[gidx] = fe - 1;
        }
      }
      n_groups = __popcll(fm);
    }
  }
  if (lane == 0) { rl.n_groups = n_groups; rl.status = status; }

  if (!commit) return;
  const LayerState& so = ra.st_out;
  const bool ok = status == MOE_OK;
  const FastTable& w = ok ? f : f0;
  if (lane < C) { so.tick[lane] = w.tick; so.expert_in[lane] = w.exp; so.buf_of_slot[lane] = w.buf; }
  if (lane < P) { so.used_stamp[lane] = w.used; so.free_buf[lane] = w.free_b; so.zombie[lane] = w.zomb; }
  if (ok && lane < n_lookups && f0.trace_n + lane < a.trace_cap)
    so.trace[f0.trace_n + lane] = moe_trace_rec_t{a.row0 + lane / K, my_e, my_hit, my_evicted};
  if (ok && lane < NP) { t.wpair[lane] = rl.wpair[lane]; t.pos_of[lane] = rank; }   // for the combine launch
  if (lane == 0) {
    so.scalars[SC_CLOCK] = w.clock;
    so.scalars[SC_NRES] = w.n_res;
    so.scalars[SC_NFREE] = w.n_free;
    so.scalars[SC_NZOMBIE] = w.n_zombie;
    so.scalars[SC_CALLSEQ] = seq;
    so.scalars[SC_TRACE_N] = f0.trace_n + (ok ? n_lookups : 0);
    if (ok) {
      ra.dev_stats[0] += (unsigned long long)n_hits;
      ra.dev_stats[1] += (unsigned long long)n_miss;
      ra.dev_stats[2] += (unsigned long long)n_evict;
    }
    auto record = [&](Mailbox* mb) {
      mb->status = status;
      mb->n_miss = n_miss;
      mb->n_evict = n_evict;
      mb->n_groups = n_groups;
      mb->n_hits = n_hits;
      mb->seq = seq;
    };
    record(a.mailbox);
    if (ra.log) record(ra.log);
  }
}

// Router logits of the call's (at most 4) tokens as one small matrix product on the matrix cores, repeated by
// every workgroup (Eq. 1): rows of W_r are the A operand, the tokens the B operand of v_mfma_f32_16x16x32_bf16.
// W_r is read from the library's own copy in operand order (pack_router_kernel below): one wave-wide load is one
// contiguous KiB, as for the expert weights; read row-major, the same fragment is 16 pieces of 64 bytes and the
// address unit of the compute unit, not the cache, sets the pace (measured: 10 us against 5 us per workgroup).
// The tokens go through LDS, so that a wave can keep 16 weight fragments in flight.  What remains (5 us for a
// 64 x 2048 matrix) is the rate at which the caches serve the same 262 KB to all 256 compute units at once, not
// latency: deeper batches, sixteen waves and touching the later fragments ahead of time all left it unchanged.  The waves split the expert
// tiles and, when there are more waves than tiles, the contraction; the slices meet in LDS (pz, WAVES x 2 x 256
// floats).
template <int WAVES>
__device__ __forceinline__ void route_logits(const RoutedArgs& ra, float* pz, RoutedLds& rl) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, q = lane >> 4;
  const int B = ra.a.B, E = ra.a.E, d = ra.r.d;
  const int nkb = d >> 5;
  const int tiles = (E + 15) >> 4;
  const int S = WAVES >= tiles ? WAVES / tiles : 1;       // contraction slices per expert tile
  const int n_items = tiles * S;                          // (tile, slice) units, dealt to the waves
  constexpr int U = 16;                                   // weight fragments a wave keeps in flight
  // the tokens: one coalesced copy into LDS, its loads issued ahead of the first weight fragments
  const int n_xv = B * d / 8;
  constexpr int kXv = (kRoutedMaxX / 8 + 64 * WAVES - 1) / (64 * WAVES);
  u32x4 xv[kXv];
#pragma unroll
  for (int i = 0; i < kXv; ++i) {
    const int v = threadIdx.x + i * 64 * WAVES;
    xv[i] = v < n_xv ? static_cast<const u32x4*>(ra.r.x)[v] : u32x4{0, 0, 0, 0};
  }
  float bv[kRoutedMaxB * kRoutedMaxE / (64 * WAVES) + 1];
#pragma unroll
  for (int i = 0; i < kRoutedMaxB * kRoutedMaxE / (64 * WAVES) + 1; ++i) {
    const int v = threadIdx.x + i * 64 * WAVES;
    bv[i] = (ra.r.bias && v < B * E) ? ra.r.bias[v] : 0.f;
  }
  int item = wave, kb0 = item / tiles;
  bool have = item < n_items;
  u32x4 wa[U];
  auto load_batch = [&]() {
    const u32x4* wfrag = static_cast<const u32x4*>(ra.router_packed) + (size_t)(item % tiles) * nkb * 64 + lane;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kb = kb0 + u * S < nkb ? kb0 + u * S : nkb - 1;    // clamped: in bounds, not used below
      wa[u] = wfrag[(size_t)kb * 64];
    }
  };
  if (have) load_batch();
#pragma unroll
  for (int i = 0; i < kXv; ++i) {
    const int v = threadIdx.x + i * 64 * WAVES;
    if (v < n_xv) rl.xs[v] = xv[i];
  }
#pragma unroll
  for (int i = 0; i < kRoutedMaxB * kRoutedMaxE / (64 * WAVES) + 1; ++i) {
    const int v = threadIdx.x + i * 64 * WAVES;
    if (v < B * E) rl.bias[v] = bv[i];
  }
  for (int e = threadIdx.x; e < E; e += 64 * WAVES) rl.buf_of[e] = -1;
  __syncthreads();
  // columns beyond the call's tokens read token 0 again: their results are never looked at
  const uint16_t* xl = reinterpret_cast<const uint16_t*>(rl.xs) + (size_t)(n < B ? n : 0) * d + q * 8;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  while (have) {        // uniform per wave
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (kb0 + u * S < nkb)      // uniform
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
            __builtin_bit_cast(bf16x8, wa[u]),
            __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xl + (size_t)(kb0 + u * S) * 32)), acc, 0, 0, 0);
    kb0 += U * S;
    if (kb0 >= nkb) {
      *reinterpret_cast<f32x4*>(pz + (size_t)item * 256 + lane * 4) = acc;
      acc = f32x4{0.f, 0.f, 0.f, 0.f};
      item += WAVES;
      kb0 = item / tiles;
      have = item < n_items;
    }
    if (have) load_batch();
  }
  __syncthreads();
  for (int i = threadIdx.x; i < B * E; i += 64 * WAVES) {
    const int b = i / E, e = i - b * E;
    const int tile = e >> 4, m = e & 15;
    const int src = ((m >> 2) * 16 + b) * 4 + (m & 3);      // where the MFMA left (expert m of the tile, token b)
    float v = 0.f;
    for (int sl = 0; sl < S; ++sl) v += pz[(size_t)(sl * tiles + tile) * 256 + src];
    rl.zs[b][e] = v + rl.bias[i];
  }
  __syncthreads();
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
  const int wave = threadIdx.x >> 6;
  const int c = blockIdx.x;  // chunk of 32 intermediate rows

  int gd_buf, gd_begin, gd_count, gd_miss, gd_expert, gd_pair0;
  if constexpr (ROUTED) {
    RoutedLds& rl = rl_store;
    const RoutedArgs& ra = *rap;
    // the row of workgroups behind the last group keeps the books: its first workgroup does what the others do,
    // plus the gate weights, the table after the call, the trace, the counters and the call record; it runs no
    // expert, so none of that delays the streaming
    const bool keeper = (int)blockIdx.y == a.g_max;
    if (keeper && blockIdx.x != 0) return;
    FastTable ft{};
    if (wave == 0) ft = fast_load(ra.st_in, ra.a.C, ra.a.P);     // in flight while the logits are formed
    int tb_exp = -1, tb_buf = -1;     // the last wave inverts the table: expert -> buffer
    if (wave == WAVES - 1 && lane < ra.a.C) { tb_exp = ra.st_in.expert_in[lane]; tb_buf = ra.st_in.buf_of_slot[lane]; }
    route_logits<WAVES>(ra, &red[0][0][0], rl);
    if (wave == WAVES - 1 && tb_exp >= 0) rl.buf_of[tb_exp] = tb_buf;
    for (int b = wave; b < ra.a.B; b += WAVES) {
      if (keeper) {
        if (ra.a.E <= 64) gate_token<1>(rl.zs[b], b, ra.a.E, ra.a.K, ra.a.KS, ra.r.norm_topk, rl.idx, rl.wpair, ra.r.user_idx, ra.r.user_w, nullptr);
        else gate_token<kRoutedMaxE / 64>(rl.zs[b], b, ra.a.E, ra.a.K, ra.a.KS, ra.r.norm_topk, rl.idx, rl.wpair, ra.r.user_idx, ra.r.user_w, nullptr);
      } else {      // only the selected set: the weights are the bookkeeper's business
        if (ra.a.E <= 64) gate_token<1, false>(rl.zs[b], b, ra.a.E, ra.a.K, ra.a.KS, 0, rl.idx, nullptr, nullptr, nullptr, nullptr);
        else gate_token<kRoutedMaxE / 64, false>(rl.zs[b], b, ra.a.E, ra.a.K, ra.a.KS, 0, rl.idx, nullptr, nullptr, nullptr, nullptr);
      }
    }
    __syncthreads();
    if (wave == 0) lookup_small(ft, rl, ra, a.t, keeper);
    if (keeper) return;
    __syncthreads();
    // (values read from LDS are the same in every lane: saying so keeps them, and the addresses formed from
    // them, in scalar registers)
    if (g >= __builtin_amdgcn_readfirstlane(rl.n_groups)) return;         // also when the call failed: nothing runs
    gd_buf = __builtin_amdgcn_readfirstlane(rl.g_buf[g]);
    gd_begin = __builtin_amdgcn_readfirstlane(rl.g_begin[g]);
    gd_count = __builtin_amdgcn_readfirstlane(rl.g_count[g]);
    gd_miss = __builtin_amdgcn_readfirstlane(rl.g_miss[g]);
    gd_expert = __builtin_amdgcn_readfirstlane(rl.g_expert[g]);
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

template <typename T>
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
      v[u] = *reinterpret_cast<const f32x4*>(o_part + ((size_t)pos_of[(size_t)b * KS + j] * n_chunks + c) * d + col);
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

bool decode_single_supported(int policy, int E, int C, int P, int n_shared, int K, int d, int f, int batch) {
  if (!fast_table(policy, C, P, n_shared)) return false;
  if (batch > kRoutedMaxB || batch * d > kRoutedMaxX || batch * (K + n_shared) > kWave || E > kRoutedMaxE) return false;
  if (!ffn_fused_supported(d, f, batch)) return false;
  const int g_max = std::min(batch * K, P) + n_shared;
  const int waves = pick_waves(d, (f / 32) * g_max);
  return waves != 0 && (E + 15) / 16 <= 2 * waves;      // the logit tiles of the waves fit their LDS scratch
}

hipError_t launch_decode_single(hipStream_t s, const FfnArgs& a, const RoutedArgs& ra, KernelEvents ev) {
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
                                 int B, int KS, int d, int n_chunks, void* y) {
  dim3 grid(B, d / (kCombLanes * 4)), block(kCombLanes * kCombSlices);
  hipLaunchKernelGGL(combine_chunks_kernel<uint16_t>, grid, block, 0, s, o_part, wpair, pos_of, KS, d, n_chunks,
                     (uint16_t*)y);
  return hipGetLastError();
}

}  // namespace moe
