// Prologue of the single-launch decode kernels (bf16 and INT4 experts): every workgroup derives the router
// logits (paper Eq. 1), the selected experts, the cache lookups and the groups of the call for itself, so that the
// expert FFN can start in the same launch without a round trip through memory or the host.
#pragma once
#include <type_traits>

#include "device_utils.hpp"
#include "gating.hpp"
#include "moe_internal.hpp"

namespace moe {

typedef __bf16 rp_bf16x8 __attribute__((ext_vector_type(8)));
typedef float rp_f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t rp_u32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------- single-launch decode: prologue pieces
// Limits of the routed variant: tokens per call, experts whose logits a workgroup keeps, token elements staged.
constexpr int kRoutedMaxB = 4, kRoutedMaxE = 256, kRoutedMaxX = 8192;

// What every workgroup of the routed variant derives for itself, in LDS.
struct RoutedLds {
  rp_u32x4 xs[kRoutedMaxX / 8];            // the call's tokens [B][d], bf16
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
__device__ inline void lookup_small(FastTable f, RoutedLds& rl, const RoutedArgs& ra, const CallTables& t, bool commit) {
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
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
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
  rp_u32x4 xv[kXv];
#pragma unroll
  for (int i = 0; i < kXv; ++i) {
    const int v = threadIdx.x + i * 64 * WAVES;
    xv[i] = v < n_xv ? static_cast<const rp_u32x4*>(ra.r.x)[v] : rp_u32x4{0, 0, 0, 0};
  }
  float bv[kRoutedMaxB * kRoutedMaxE / (64 * WAVES) + 1];
#pragma unroll
  for (int i = 0; i < kRoutedMaxB * kRoutedMaxE / (64 * WAVES) + 1; ++i) {
    const int v = threadIdx.x + i * 64 * WAVES;
    bv[i] = (ra.r.bias && v < B * E) ? ra.r.bias[v] : 0.f;
  }
  int item = wave, kb0 = item / tiles;
  bool have = item < n_items;
  rp_u32x4 wa[U];
  auto load_batch = [&]() {
    const rp_u32x4* wfrag = static_cast<const rp_u32x4*>(ra.router_packed) + (size_t)(item % tiles) * nkb * 64 + lane;
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
  rp_f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  while (have) {        // uniform per wave
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (kb0 + u * S < nkb)      // uniform
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
            __builtin_bit_cast(rp_bf16x8, wa[u]),
            __builtin_bit_cast(rp_bf16x8, *reinterpret_cast<const rp_u32x4*>(xl + (size_t)(kb0 + u * S) * 32)), acc, 0, 0, 0);
    kb0 += U * S;
    if (kb0 >= nkb) {
      *reinterpret_cast<rp_f32x4*>(pz + (size_t)item * 256 + lane * 4) = acc;
      acc = rp_f32x4{0.f, 0.f, 0.f, 0.f};
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


// The group a workgroup of the expert phase works on.
struct GroupView { int buf, begin, count, miss, expert; };

// Runs the prologue in the calling workgroup (all waves must call it).  pz: LDS scratch of WAVES x 2 x 256 floats.
// g_max: number of group rows of the grid; the row behind them keeps the books (its first workgroup does what the
// others do, plus the gate weights, the table after the call, the trace, the counters and the call record; it
// runs no expert, so none of that delays the streaming).  Returns false when the workgroup has nothing to
// stream: the bookkeeping row, rows beyond the call's groups, a call that failed.
template <int WAVES>
__device__ __forceinline__ bool routed_prologue(const FfnArgs& a, const RoutedArgs& ra, RoutedLds& rl, float* pz,
                                                GroupView& gd) {
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int g = blockIdx.y;
  const bool keeper = g == a.g_max;
  if (keeper && blockIdx.x != 0) return false;
  FastTable ft{};
  if (wave == 0) ft = fast_load(ra.st_in, ra.a.C, ra.a.P);     // in flight while the logits are formed
  int tb_exp = -1, tb_buf = -1;     // the last wave inverts the table: expert -> buffer
  if (wave == WAVES - 1 && lane < ra.a.C) { tb_exp = ra.st_in.expert_in[lane]; tb_buf = ra.st_in.buf_of_slot[lane]; }
  route_logits<WAVES>(ra, pz, rl);
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
  if (keeper) return false;
  __syncthreads();
  // (values read from LDS are the same in every lane: saying so keeps them, and the addresses formed from
  // them, in scalar registers)
  if (g >= __builtin_amdgcn_readfirstlane(rl.n_groups)) return false;      // also when the call failed: nothing runs
  gd.buf = __builtin_amdgcn_readfirstlane(rl.g_buf[g]);
  gd.begin = __builtin_amdgcn_readfirstlane(rl.g_begin[g]);
  gd.count = __builtin_amdgcn_readfirstlane(rl.g_count[g]);
  gd.miss = __builtin_amdgcn_readfirstlane(rl.g_miss[g]);
  gd.expert = __builtin_amdgcn_readfirstlane(rl.g_expert[g]);
  return true;
}

}  // namespace moe
