// Router GEMV + softmax/Top-K gating + expert-cache lookup in ONE launch.
//
// Paper section 2: Eq. 1 (p = softmax(W_r x), r = Top-K(p)) and the gate
// weights of Eq. 2; then the offloading runtime of section 2 ("Expert
// Offloading Systems") and section 3.2: a selected expert that is not resident
// is fetched on demand and a cached expert is evicted as the policy dictates.
// LRU is the gamma -> 0+ member and LFU the gamma = 1 member of the
// discounted-count family of Definition C.1; contents change lazily, only by
// inserting the requested expert (Remark after Definition C.1).
//
// Shape of the launch: one workgroup per token.
//   phase 1: the waves of the workgroup split the E router rows; each wave forms
//     whole dot products W_r[e,:].x for up to four rows at a time with every
//     16-byte load issued up front, then DPP reductions.  Logits stay in LDS.
//   phase 2: wave 0 owns the token: Top-K by K rounds of wave arg-max on the
//     logits (ties to the lower id; the same set as Top-K of p), softmax with
//     wave reductions, gate weights, outputs in ascending expert id.
//   phase 3 (the only workgroup, or for a batch the one that arrives last at a
//     device-scope counter - nobody waits): ONE wave runs the B*K lookups in
//     order, since each one changes the state the next one sees.  For the
//     usual sizes (LRU, at most 64 slots/buffers/pairs) the whole table lives
//     in registers, one slot per lane, and a lookup is a ballot plus a DPP
//     arg-min; otherwise the table is staged in LDS.  The wave also groups the
//     (token, expert) pairs by expert buffer for the FFN kernels and leaves the
//     miss list in pinned host memory for the copy scheduler.
// Nothing is committed when the call runs out of spare buffers, so a failed call
// leaves the cache unchanged.
#include "device_utils.hpp"
#include "gating.hpp"
#include "moe_internal.hpp"

namespace moe {


namespace {

// ---------------------------------------------------------------- dot products
template <typename T> struct Vec;
template <> struct Vec<float> {
  static constexpr int N = 4;
  using type = float4;
  static __device__ __forceinline__ float dot(const float4& a, const float4& b, float acc) {
    acc = fmaf(a.x, b.x, acc); acc = fmaf(a.y, b.y, acc);
    acc = fmaf(a.z, b.z, acc); acc = fmaf(a.w, b.w, acc);
    return acc;
  }
};
template <> struct Vec<uint16_t> {
  static constexpr int N = 8;
  using type = uint4;
  static __device__ __forceinline__ float dot(const uint4& a, const uint4& b, float acc) {
    const uint32_t av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc = fmaf(__builtin_bit_cast(float, av[i] << 16), __builtin_bit_cast(float, bv[i] << 16), acc);
      acc = fmaf(__builtin_bit_cast(float, av[i] & 0xffff0000u),
                 __builtin_bit_cast(float, bv[i] & 0xffff0000u), acc);
    }
    return acc;
  }
};

constexpr int kTileMaxE = 256;   // most experts the 16-token tile kernel keeps logits for

// ---------------------------------------------------------------- LDS layout
struct LdsLayout {
  size_t tick, score, expert_in, buf_of_slot, slot_of, free_buf, zombie, used, filled, pending, count, start,
      logit, idx_stage, pair_stage, total;
};

__host__ __device__ inline bool stage_in_lds(int B, int KS) { return (size_t)B * KS <= kStageMaxPairs; }

__host__ __device__ inline LdsLayout lds_layout(int E, int C, int P, int n_shared, int B, int K, int KS) {
  LdsLayout l;
  size_t o = 0;
  l.tick = o; o += (size_t)C * 8;
  l.score = o; o += (size_t)E * 8;
  l.expert_in = o; o += (size_t)C * 4;
  l.buf_of_slot = o; o += (size_t)C * 4;
  l.slot_of = o; o += (size_t)E * 4;
  l.free_buf = o; o += (size_t)P * 4;
  l.zombie = o; o += (size_t)P * 4;
  l.used = o; o += (size_t)P * 4;
  l.filled = o; o += (size_t)P * 4;
  l.pending = o; o += (size_t)E * 4;
  const int n_keys = (P > E ? P : E) + n_shared;     // grouping keys: buffer ids, or expert ids when streaming a prompt
  l.count = o; o += (size_t)n_keys * 4;
  l.start = o; o += (size_t)n_keys * 4;
  l.logit = o; o += (size_t)E * 4;
  const bool stage = stage_in_lds(B, KS);
  l.idx_stage = o; o += stage ? (size_t)B * K * 4 : 0;
  l.pair_stage = o; o += stage ? (size_t)B * KS * 4 : 0;
  l.total = o;
  return l;
}

// ---------------------------------------------------------------- grouping (any number of pairs)
// Counting sort of the (token, expert) pairs by the buffer they read, run by ONE wave with counters in LDS.
// pair_buf[B*KS] must hold the buffer of every routed pair; shared-expert pairs are filled in here.
// The order of the pairs inside a group is whatever order the LDS atomics resolve in; every pair's arithmetic is
// independent of its position, so the layer output does not depend on it.
__device__ int group_pairs_lds(int32_t* count, int32_t* cursor, const int32_t* filled, int32_t* pair_buf,
                               const CallTables& t, const CacheCallArgs& a) {
  const int lane = threadIdx.x & 63;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  const int K = a.K, KS = a.KS, P = a.P;
  const int NP = a.B * KS, NB = P + a.n_shared;
  for (int p = lane; p < a.B * a.n_shared; p += kWave) {
    const int b = p / a.n_shared, sidx = p - b * a.n_shared;
    pair_buf[(size_t)b * KS + K + sidx] = P + sidx;
  }
  for (int i = lane; i < NB; i += kWave) count[i] = 0;
  wave_sync();
  for (int p = lane; p < NP; p += kWave) atomicAdd(&count[pair_buf[p]], 1);
  wave_sync();
  int n_groups = 0, offset = 0;
  for (int base = 0; base < NB; base += kWave) {        // ids in ascending order, 64 at a time
    const int id = base + lane;
    const int c = id < NB ? count[id] : 0;
    int incl = c;                                       // inclusive prefix sum over the lanes
#pragma unroll
    for (int dlt = 1; dlt < kWave; dlt <<= 1) {
      const int v = __shfl_up(incl, dlt);
      if (lane >= dlt) incl += v;
    }
    const int begin = offset + incl - c;
    const uint64_t gm = __ballot(c > 0);
    if (c > 0) {
      GroupDesc gd;
      const int fe = id < P ? filled[id] : 0;        // expert + 1 of a buffer being filled by this call
      gd.buf = id; gd.begin = begin; gd.count = c; gd.miss = fe != 0;
      gd.pair0 = 0; gd.expert = fe - 1; gd.pad[0] = gd.pad[1] = 0;
      t.grp[n_groups + __popcll(gm & lt_mask)] = gd;
    }
    if (id < NB) cursor[id] = begin;
    n_groups += __popcll(gm);
    offset += __shfl(incl, kWave - 1);
  }
  wave_sync();
  for (int p = lane; p < NP; p += kWave) {
    const int pos = atomicAdd(&cursor[pair_buf[p]], 1);
    t.sorted_pair[pos] = p;
    t.pos_of[p] = pos;
  }
  wave_sync();
  for (int gi = lane; gi < n_groups; gi += kWave) t.grp[gi].pair0 = t.sorted_pair[t.grp[gi].begin];
  return n_groups;
}

// ---------------------------------------------------------------- prompt streaming
// Phase 3 of a prefill call: the cache is only READ.  Pairs are grouped by expert; a group whose expert is
// resident reads its buffer, any other group streams its expert from the pinned host pool (miss = 1) and
// nothing is inserted or refreshed, so a one-off scan over a long prompt leaves the cache as the prefetch set
// it.  Runs in ONE wave; idx [B][K] routed experts (LDS or global), keys [B*KS] scratch.
__device__ void prefill_phase(unsigned char* smem, const LdsLayout& L, const int32_t* idx, int32_t* keys,
                              const LayerState& st, const CallTables& t, const CacheCallArgs& a) {
  int32_t* slot_of = reinterpret_cast<int32_t*>(smem + L.slot_of);
  int32_t* count = reinterpret_cast<int32_t*>(smem + L.count);
  int32_t* cursor = reinterpret_cast<int32_t*>(smem + L.start);
  const int lane = threadIdx.x & 63;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  const int E = a.E, C = a.C, K = a.K, KS = a.KS, P = a.P;
  const int NP = a.B * KS, NB = E + a.n_shared;
  for (int e = lane; e < E; e += kWave) slot_of[e] = -1;
  for (int i = lane; i < NB; i += kWave) count[i] = 0;
  wave_sync();
  for (int s = lane; s < C; s += kWave) {
    const int ex = st.expert_in[s];
    if (ex >= 0) slot_of[ex] = st.buf_of_slot[s];          // expert -> the buffer that holds it
  }
  for (int p = lane; p < NP; p += kWave) {
    const int b = p / KS, k = p - b * KS;
    keys[p] = k < K ? idx[(size_t)b * K + k] : E + (k - K);
  }
  wave_sync();
  for (int p = lane; p < NP; p += kWave) atomicAdd(&count[keys[p]], 1);
  wave_sync();
  int n_groups = 0, offset = 0, n_stream = 0;
  for (int base = 0; base < NB; base += kWave) {
    const int id = base + lane;
    const int c = id < NB ? count[id] : 0;
    int incl = c;
#pragma unroll
    for (int dlt = 1; dlt < kWave; dlt <<= 1) {
      const int v = __shfl_up(incl, dlt);
      if (lane >= dlt) incl += v;
    }
    const int begin = offset + incl - c;
    const uint64_t gm = __ballot(c > 0);
    const int buf = id < E ? slot_of[id < E ? id : 0] : P + (id - E);
    const bool streamed = c > 0 && id < E && buf < 0;
    if (c > 0) {
      GroupDesc gd;
      gd.buf = streamed ? 0 : buf; gd.begin = begin; gd.count = c; gd.miss = streamed ? 1 : 0;
      gd.pair0 = 0; gd.expert = streamed ? id : -1; gd.pad[0] = gd.pad[1] = 0;
      t.grp[n_groups + __popcll(gm & lt_mask)] = gd;
    }
    if (id < NB) cursor[id] = begin;
    n_groups += __popcll(gm);
    n_stream += __popcll(__ballot(streamed));
    offset += __shfl(incl, kWave - 1);
  }
  wave_sync();
  for (int p = lane; p < NP; p += kWave) {
    const int pos = atomicAdd(&cursor[keys[p]], 1);
    t.sorted_pair[pos] = p;
    t.pos_of[p] = pos;
  }
  wave_sync();
  for (int gi = lane; gi < n_groups; gi += kWave) t.grp[gi].pair0 = t.sorted_pair[t.grp[gi].begin];
  if (lane == 0) {
    *t.n_groups = n_groups;
    Mailbox* mb = a.mailbox;
    mb->status = MOE_OK;
    mb->n_miss = n_stream;
    mb->n_evict = 0;
    mb->n_groups = n_groups;
    mb->n_hits = 0;
    mb->seq = a.seq;
  }
}

// ---------------------------------------------------------------- phase 3
// General path (any C, P, batch; both policies): the table lives in LDS.
// Runs in ONE wave.  idx: selected experts [B][K] (LDS or global); pair_buf: scratch [B*KS].
__device__ void cache_phase_general(unsigned char* smem, const LdsLayout& L, const int32_t* idx, int32_t* pair_buf,
                            const LayerState& st, const CallTables& t, const CacheCallArgs& a) {
  uint64_t* tick = reinterpret_cast<uint64_t*>(smem + L.tick);
  double* score = reinterpret_cast<double*>(smem + L.score);
  int32_t* expert_in = reinterpret_cast<int32_t*>(smem + L.expert_in);
  int32_t* buf_of_slot = reinterpret_cast<int32_t*>(smem + L.buf_of_slot);
  int32_t* slot_of = reinterpret_cast<int32_t*>(smem + L.slot_of);
  int32_t* free_buf = reinterpret_cast<int32_t*>(smem + L.free_buf);
  int32_t* zombie = reinterpret_cast<int32_t*>(smem + L.zombie);
  uint32_t* used = reinterpret_cast<uint32_t*>(smem + L.used);
  int32_t* filled = reinterpret_cast<int32_t*>(smem + L.filled);
  int32_t* pending = reinterpret_cast<int32_t*>(smem + L.pending);
  int32_t* count = reinterpret_cast<int32_t*>(smem + L.count);
  int32_t* start = reinterpret_cast<int32_t*>(smem + L.start);

  const int lane = threadIdx.x & 63;
  const int E = a.E, C = a.C, P = a.P, K = a.K, KS = a.KS;
  const bool gamma_policy = a.policy == MOE_POLICY_GAMMA;

  // ---- load the table (independent loads, one round trip) ----
  int64_t clock = st.scalars[SC_CLOCK];
  int n_res = (int)st.scalars[SC_NRES];
  int n_free = (int)st.scalars[SC_NFREE];
  int n_zombie = (int)st.scalars[SC_NZOMBIE];
  const int64_t trace_n = st.scalars[SC_TRACE_N];
  for (int s = lane; s < C; s += kWave) {
    tick[s] = st.tick[s]; expert_in[s] = st.expert_in[s]; buf_of_slot[s] = st.buf_of_slot[s];
  }
  for (int e = lane; e < E; e += kWave) {
    slot_of[e] = -1; pending[e] = 0;
    if (gamma_policy) score[e] = st.score[e];
  }
  for (int i = lane; i < P; i += kWave) {
    used[i] = st.used_stamp[i]; filled[i] = 0;
    // free stack, then the buffers the previous call released (all its kernels have finished)
    if (i < n_free) free_buf[i] = st.free_buf[i];
    else if (i < n_free + n_zombie) free_buf[i] = st.zombie[i - n_free];
  }
  n_free += n_zombie;
  n_zombie = 0;
  wave_sync();
  for (int s = lane; s < C; s += kWave)       // expert -> slot index, rebuilt from the slots
    if (expert_in[s] >= 0) slot_of[expert_in[s]] = s;
  wave_sync();

  const uint32_t seq = a.seq;
  const int n_lookups = a.mode == 0 ? a.B * K : K;
  int status = MOE_OK, n_miss = 0, n_evict = 0, n_hits = 0;
  int64_t trace_added = 0;

  for (int q = 0; q < n_lookups; ++q) {
    const int b = a.mode == 0 ? q / K : 0;
    const int k = a.mode == 0 ? q % K : q;
    const int e = a.mode == 0 ? idx[q] : a.pin_ids[q];
    int s = slot_of[e];
    int evicted = -1, buf;
    const bool hit = s >= 0;
    if (hit) {
      buf = buf_of_slot[s];
      ++n_hits;
    } else {
      if (n_res < C) {            // slots fill in index order, so the lowest empty slot is n_res
        s = n_res;
        buf = free_buf[n_free - 1];
        --n_free;
        ++n_res;
      } else {
        int vs = -1;
        uint64_t vt = ~0ull;
        double vsc = 0.0;
        for (int c = lane; c < C; c += kWave) {
          const uint64_t tc = tick[c];
          if (!gamma_policy) {
            if (tc < vt) { vt = tc; vs = c; }
          } else {
            const int ex = expert_in[c];
            if (pending[ex]) continue;     // wanted by the current token: never a victim
            const double sc = score[ex];
            if (vs < 0 || sc < vsc || (sc == vsc && tc < vt)) { vsc = sc; vt = tc; vs = c; }
          }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
          const int os = __shfl_xor(vs, off);
          const uint64_t ot = __shfl_xor((unsigned long long)vt, off);
          const double osc = __shfl_xor(vsc, off);
          bool take;
          if (os < 0) take = false;
          else if (vs < 0) take = true;
          else if (!gamma_policy) take = ot < vt;
          else take = osc < vsc || (osc == vsc && ot < vt);
          if (take) { vs = os; vt = ot; vsc = osc; }
        }
        s = vs;
        evicted = expert_in[s];
        const int vb = buf_of_slot[s];
        if (used[vb] == seq) {    // an earlier token of this call reads that buffer: leave it intact
          if (n_free == 0) { status = MOE_ERR_STAGING_EXHAUSTED; break; }
          buf = free_buf[n_free - 1];
          --n_free;
          if (lane == 0) zombie[n_zombie] = vb;
          ++n_zombie;
        } else {
          buf = vb;
        }
        ++n_evict;
      }
      if (lane == 0) {
        if (evicted >= 0) slot_of[evicted] = -1;
        expert_in[s] = e;
        slot_of[e] = s;
        buf_of_slot[s] = buf;
        filled[buf] = e + 1;
        if (n_miss < a.max_miss) a.miss_list[n_miss] = MissEntry{e, buf};
      }
      ++n_miss;
    }
    ++clock;
    if (lane == 0) {
      tick[s] = (uint64_t)clock;
      used[buf] = seq;
      pending[e] = 1;
      if (a.mode == 0) {
        pair_buf[(size_t)b * KS + k] = buf;
        if (trace_n + trace_added < a.trace_cap)
          st.trace[trace_n + trace_added] = moe_trace_rec_t{a.row0 + b, e, hit ? 1 : 0, evicted};
      }
    }
    if (a.mode == 0) ++trace_added;
    wave_sync();
    // Definition C.1: the discounted counts advance once per token (each pinned expert is a token)
    if (gamma_policy && (a.mode == 1 || k == K - 1)) {
      for (int x = lane; x < E; x += kWave) {
        score[x] = __dadd_rn(__dmul_rn(a.gamma, score[x]), (double)pending[x]);
        pending[x] = 0;
      }
      wave_sync();
    }
  }
  int n_groups = 0;
  if (status == MOE_OK && a.mode == 0) {
    n_groups = group_pairs_lds(count, start, filled, pair_buf, t, a);
  }
  if (a.mode == 0 && lane == 0) *t.n_groups = n_groups;

  if (status == MOE_OK) {
    // ---- commit ----
    wave_sync();
    for (int s = lane; s < C; s += kWave) {
      st.tick[s] = tick[s]; st.expert_in[s] = expert_in[s]; st.buf_of_slot[s] = buf_of_slot[s];
    }
    if (gamma_policy)
      for (int e = lane; e < E; e += kWave) st.score[e] = score[e];
    for (int i = lane; i < n_free; i += kWave) st.free_buf[i] = free_buf[i];
    for (int i = lane; i < n_zombie; i += kWave) st.zombie[i] = zombie[i];
    for (int i = lane; i < P; i += kWave) st.used_stamp[i] = used[i];
    if (lane == 0) {
      st.scalars[SC_CLOCK] = clock;
      st.scalars[SC_NRES] = n_res;
      st.scalars[SC_NFREE] = n_free;
      st.scalars[SC_NZOMBIE] = n_zombie;
      st.scalars[SC_CALLSEQ] = seq;
      st.scalars[SC_TRACE_N] = trace_n + trace_added;
    }
  }
  if (lane == 0) {
    Mailbox* mb = a.mailbox;
    mb->status = status;
    mb->n_miss = n_miss;
    mb->n_evict = n_evict;
    mb->n_groups = n_groups;
    mb->n_hits = n_hits;
    mb->seq = seq;   // read by the host only after the kernel has completed
  }
}

// Runs in ONE wave.  idx_src: the experts to look up, in order (decode: [B][K]; pin: the list);
// pair_buf: scratch [B*KS] (LDS or global), used when the call has more than 64 pairs.
__device__ void cache_phase_fast(FastTable f, unsigned char* smem, const LdsLayout& L, const int32_t* idx_src,
                                 int32_t* pair_buf, const LayerState& st, const CallTables& t,
                                 const CacheCallArgs& a) {
  const int lane = threadIdx.x & 63;
  const int C = a.C, P = a.P, K = a.K, KS = a.KS;
  // LDS scratch (the table itself lives in registers on this path)
  int32_t* lds_slot_of = reinterpret_cast<int32_t*>(smem + L.slot_of);     // [E] expert -> slot
  int32_t* lds_last = reinterpret_cast<int32_t*>(smem + L.free_buf);       // [P >= C] last lookup of a slot, +1
  int32_t* lds_touch = reinterpret_cast<int32_t*>(smem + L.zombie);        // [P] buffer read by the chunk
  int32_t* lds_filled = reinterpret_cast<int32_t*>(smem + L.filled);       // [P]
  int32_t* lds_count = reinterpret_cast<int32_t*>(smem + L.count);         // [P + n_shared]
  int32_t* lds_cursor = reinterpret_cast<int32_t*>(smem + L.start);        // [P + n_shared]
  // buffers released by the previous call: all its kernels have finished, reuse them
  {
    const int src = lane - f.n_free;
    const int z = __shfl(f.zomb, src < 0 ? 0 : src);
    if (src >= 0 && src < f.n_zombie) f.free_b = z;
    f.n_free += f.n_zombie;
    f.n_zombie = 0;
  }
  const uint32_t seq = a.seq;
  const int n_lookups = a.mode == 0 ? a.B * K : K;
  const int NP = a.B * KS;
  const bool small = NP <= kWave;     // all pairs fit one per lane
  int status = MOE_OK, n_miss = 0, n_evict = 0, n_hits = 0;
  int my_pair = -1;       // small calls: lane p = b*KS + k holds the buffer the pair reads
  int filled = 0;         // lane p: expert + 1 that this call brings into buffer p, 0 if none

  // ---- shortcut for a call whose lookups all hit (the resident regime): residency does not change, and the
  //      recency updates commute - the last lookup of a slot decides its tick.  Lookups run 64 per step. ----
  bool all_hit = false;
  if (a.mode == 0 && f.n_res > 0 && n_lookups >= 16) {     // a handful of lookups takes the register variant below
    for (int e = lane; e < a.E; e += kWave) lds_slot_of[e] = -1;
    if (lane < P) { lds_last[lane] = 0; lds_touch[lane] = 0; }
    wave_sync();
    if (lane < C && f.exp >= 0) lds_slot_of[f.exp] = lane;
    wave_sync();
    uint64_t any_miss = 0;
    for (int chunk0 = 0; chunk0 < n_lookups; chunk0 += kWave) {
      const bool valid = chunk0 + lane < n_lookups;
      any_miss |= __ballot(valid && lds_slot_of[idx_src[chunk0 + lane]] < 0);
    }
    all_hit = any_miss == 0;
  }
  // the same shortcut for a handful of lookups (one per lane), entirely in registers: nothing is changed
  // unless every lookup hits
  if (a.mode == 0 && f.n_res > 0 && n_lookups < 16 && small) {
    const int my_e = lane < n_lookups ? idx_src[lane] : -3;
    int my_slot = 0;
    uint64_t new_tick = f.tick;
    bool ok = true;
    for (int q = 0; q < n_lookups; ++q) {       // uniform
      const uint64_t hm = __ballot(f.exp == readlane_i(my_e, q));
      if (hm == 0) { ok = false; break; }
      const int s = __ffsll((unsigned long long)hm) - 1;
      if (lane == q) my_slot = s;
      if (lane == s) new_tick = (uint64_t)(f.clock + q + 1);    // the last lookup of a slot decides its tick
    }
    if (ok) {
      f.tick = new_tick;
      const int my_buf = __shfl(f.buf, my_slot);                // lane q: buffer that lookup q reads
      for (int q = 0; q < n_lookups; ++q)
        if (lane == readlane_i(my_buf, q)) f.used = seq;
      if (lane < n_lookups && f.trace_n + lane < a.trace_cap)
        st.trace[f.trace_n + lane] = moe_trace_rec_t{a.row0 + lane / K, my_e, 1, -1};
      const int b = lane / KS, k = lane - b * KS;
      const int v = __shfl(my_buf, k < K ? b * K + k : 0);
      if (lane < NP && k < K) my_pair = v;
      f.clock += n_lookups;
      n_hits = n_lookups;
      all_hit = true;
    }
  } else if (all_hit) {
    for (int chunk0 = 0; chunk0 < n_lookups; chunk0 += kWave) {
      const int l = chunk0 + lane;
      const bool valid = l < n_lookups;
      const int my_e = valid ? idx_src[l] : 0;
      const int my_slot = valid ? lds_slot_of[my_e] : 0;
      if (valid) atomicMax(&lds_last[my_slot], l + 1);
      const int my_buf = __shfl(f.buf, my_slot);
      if (valid && f.trace_n + l < a.trace_cap) st.trace[f.trace_n + l] = moe_trace_rec_t{a.row0 + l / K, my_e, 1, -1};
      if (small) {
        // lane p = b*KS + k takes the buffer of lookup b*K + k (a single step)
        const int b = lane / KS, k = lane - b * KS;
        const int v = __shfl(my_buf, k < K ? b * K + k : 0);
        if (lane < NP && k < K) my_pair = v;
      } else if (valid) {
        const int b = l / K;
        pair_buf[(size_t)b * KS + (l - b * K)] = my_buf;
      }
    }
    wave_sync();
    const int last = lane < C ? lds_last[lane] : 0;
    if (last > 0) {
      f.tick = (uint64_t)(f.clock + last);
      lds_touch[f.buf] = 1;
    }
    wave_sync();
    if (lane < P && lds_touch[lane]) f.used = seq;
    f.clock += n_lookups;
    n_hits = n_lookups;
  }

  for (int chunk0 = 0; chunk0 < n_lookups && status == MOE_OK && !all_hit; chunk0 += kWave) {
    const int nl = min(kWave, n_lookups - chunk0);
    const int my_e = lane < nl ? idx_src[chunk0 + lane] : -3;
    int my_buf = -1;      // lane q: buffer that lookup chunk0 + q reads
    {
      for (int q = 0; q < nl; ++q) {
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
          if (lane == 0 && n_miss < a.max_miss) a.miss_list[n_miss] = MissEntry{e, buf};
          ++n_miss;
        }
        ++f.clock;
        if (lane == s) f.tick = (uint64_t)f.clock;
        if (lane == buf) f.used = seq;
        if (lane == q) my_buf = buf;
        if (a.mode == 0 && lane == 0 && f.trace_n + chunk0 + q < a.trace_cap)
          st.trace[f.trace_n + chunk0 + q] = moe_trace_rec_t{a.row0 + (chunk0 + q) / K, e, hit ? 1 : 0, evicted};
      }
    }
    if (a.mode == 0 && status == MOE_OK) {
      if (small) {
        // lane p = b*KS + k takes the buffer of lookup b*K + k (a single chunk)
        const int b = lane / KS, k = lane - b * KS;
        const int v = __shfl(my_buf, k < K ? b * K + k : 0);
        if (lane < NP && k < K) my_pair = v;
      } else if (lane < nl) {
        const int l = chunk0 + lane, b = l / K;
        pair_buf[(size_t)b * KS + (l - b * K)] = my_buf;
      }
    }
  }

  int n_groups = 0;
  if (status == MOE_OK && a.mode == 0) {
    if (small) {
      // ---- group the pairs by buffer: rank every pair against all others (stable) ----
      {
        const int b = lane / KS, k = lane - b * KS;
        if (lane < NP && k >= K) my_pair = P + (k - K);     // shared experts
      }
      int rank = 0, same_before = 0, cnt = 0;
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
      const int was_filled = __shfl(filled, my_pair < P && my_pair >= 0 ? my_pair : 0);
      if (lane < NP) {
        t.sorted_pair[rank] = lane;
        t.pos_of[lane] = rank;
        if (is_first) {
          GroupDesc gd;
          const int fe = my_pair < P ? was_filled : 0;
          gd.buf = my_pair; gd.begin = rank; gd.count = cnt; gd.miss = fe != 0;
          gd.pair0 = lane;      // stable order: the group's first pair is its lowest pair id
          gd.expert = fe - 1; gd.pad[0] = gd.pad[1] = 0;
          t.grp[gidx] = gd;
        }
      }
      n_groups = __popcll(fm);
    } else {
      // ---- more than 64 pairs: counting sort with the counters in LDS ----
      if (lane < P) lds_filled[lane] = filled;
      wave_sync();
      n_groups = group_pairs_lds(lds_count, lds_cursor, lds_filled, pair_buf, t, a);
    }
  }
  if (a.mode == 0 && lane == 0) *t.n_groups = n_groups;

  if (status == MOE_OK) {
    // ---- commit ----
    if (lane < C) { st.tick[lane] = f.tick; st.expert_in[lane] = f.exp; st.buf_of_slot[lane] = f.buf; }
    if (lane < P) { st.used_stamp[lane] = f.used; st.free_buf[lane] = f.free_b; st.zombie[lane] = f.zomb; }
    if (lane == 0) {
      st.scalars[SC_CLOCK] = f.clock;
      st.scalars[SC_NRES] = f.n_res;
      st.scalars[SC_NFREE] = f.n_free;
      st.scalars[SC_NZOMBIE] = f.n_zombie;
      st.scalars[SC_CALLSEQ] = seq;
      st.scalars[SC_TRACE_N] = f.trace_n + (a.mode == 0 ? n_lookups : 0);
    }
  }
  if (lane == 0) {
    Mailbox* mb = a.mailbox;
    mb->status = status;
    mb->n_miss = n_miss;
    mb->n_evict = n_evict;
    mb->n_groups = n_groups;
    mb->n_hits = n_hits;
    mb->seq = seq;   // read by the host only after the kernel has completed
  }
}

// ---------------------------------------------------------------- the decode launch
// EB: router rows a wave handles at a time (1 when there are at least as many waves as experts: no spare loads).
template <typename T, int EB>
__global__ void __launch_bounds__(1024) route_cache_kernel(RouteArgs r, LayerState st, CallTables t, CacheCallArgs a) {
  extern __shared__ __align__(8) unsigned char smem[];
  __shared__ int s_last;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int n_waves = blockDim.x >> 6;
  const int b = blockIdx.x;
  const int E = a.E, K = a.K, KS = a.KS, d = r.d;
  const bool single = gridDim.x == 1;
  const bool fast = a.mode != 2 && fast_table(a.policy, a.C, a.P, a.n_shared);

  // With one workgroup the cache table can be fetched while the router GEMV runs.
  FastTable ft{};
  if (single && fast && wave == 0) ft = fast_load(st, a.C, a.P);

  const LdsLayout L = lds_layout(E, a.C, a.P, a.n_shared, a.B, K, KS);
  float* zs = reinterpret_cast<float*>(smem + L.logit);
  const bool stage = stage_in_lds(a.B, KS);
  int32_t* idx_stage = stage ? reinterpret_cast<int32_t*>(smem + L.idx_stage) : nullptr;
  int32_t* pair_stage = stage ? reinterpret_cast<int32_t*>(smem + L.pair_stage) : t.pair_buf;

  // ---- phase 1: router rows of token b, EB rows per wave at a time ----
  {
    using V = Vec<T>;
    const int n_vec = d / V::N;  // host guarantees d % V::N == 0
    const typename V::type* xv = reinterpret_cast<const typename V::type*>(static_cast<const T*>(r.x) + (size_t)b * d);
    const typename V::type* wbase = reinterpret_cast<const typename V::type*>(r.router_w);
    for (int e0 = wave; e0 < E; e0 += n_waves * EB) {
      const typename V::type* wv[EB];
#pragma unroll
      for (int j = 0; j < EB; ++j) {
        const int e = e0 + j * n_waves;
        wv[j] = wbase + (size_t)(e < E ? e : E - 1) * n_vec;   // clamped: loads stay unconditional
      }
      float acc[EB];
#pragma unroll
      for (int j = 0; j < EB; ++j) acc[j] = 0.f;
      constexpr int CB = 4;   // chunks per lane fetched together: (1 + EB) * CB loads in flight
      for (int c0 = lane; c0 < n_vec; c0 += kWave * CB) {
        typename V::type xc[CB], wc[EB][CB];
#pragma unroll
        for (int i = 0; i < CB; ++i) {
          const int c = c0 + i * kWave;
          const int cc = c < n_vec ? c : n_vec - 1;     // clamped: in bounds, masked below
          xc[i] = xv[cc];
#pragma unroll
          for (int j = 0; j < EB; ++j) wc[j][i] = wv[j][cc];
        }
#pragma unroll
        for (int i = 0; i < CB; ++i) {
          if (c0 + i * kWave < n_vec) {
#pragma unroll
            for (int j = 0; j < EB; ++j) acc[j] = V::dot(wc[j][i], xc[i], acc[j]);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < EB; ++j) {
        const int e = e0 + j * n_waves;
        const float s = wave_sum(acc[j]);
        if (lane == 0 && e < E) zs[e] = s + (r.bias ? r.bias[(size_t)b * E + e] : 0.f);
      }
    }
  }
  __syncthreads();

  // ---- phase 2: gating of token b by wave 0 ----
  if (wave != 0) return;
  if (E <= 64) gate_token<1>(zs, b, E, K, KS, r.norm_topk, t.idx, t.wpair, r.user_idx, r.user_w, idx_stage);
  else if (E <= 256) gate_token<4>(zs, b, E, K, KS, r.norm_topk, t.idx, t.wpair, r.user_idx, r.user_w, idx_stage);
  else gate_token<16>(zs, b, E, K, KS, r.norm_topk, t.idx, t.wpair, r.user_idx, r.user_w, idx_stage);

  if (!single) {
    // ---- the last workgroup to arrive carries on (no waiting anywhere) ----
    // every lane publishes its own stores (routing results) before lane 0 announces the workgroup
    __threadfence();
    if (lane == 0) s_last = atomicAdd(r.arrive, 1) == (int)gridDim.x - 1;
    wave_sync();
    if (!s_last) return;
    if (lane == 0) __hip_atomic_store(r.arrive, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch on this stream
    __threadfence();
    // routing results of the other workgroups: read at device scope
    if (stage)
      for (int i = lane; i < a.B * K; i += kWave)
        idx_stage[i] = __hip_atomic_load(&t.idx[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (fast) ft = fast_load(st, a.C, a.P);
  }
  wave_sync();

  // ---- phase 3: cache lookups, one wave ----
  if (a.mode == 2) {
    prefill_phase(smem, L, stage ? idx_stage : t.idx, pair_stage, st, t, a);
  } else if (fast) {
    cache_phase_fast(ft, smem, L, stage ? idx_stage : t.idx, pair_stage, st, t, a);
  } else {
    cache_phase_general(smem, L, stage ? idx_stage : t.idx, pair_stage, st, t, a);
  }
}


// ---------------------------------------------------------------- many tokens per call
// Phase 3 for a large call, run by ALL waves of the last workgroup (register-table case, LRU).  The common case of
// such a call - every lookup hits - is embarrassingly parallel: residency does not change, a slot's new tick is
// the position of its last lookup (LDS atomic max), and the pairs are grouped by a counting sort with the
// counters in LDS.  A call with at least one miss hands over to the in-order routine in wave 0.
__device__ void cache_phase_fast_wide(unsigned char* smem, const LdsLayout& L, const int32_t* idx, int32_t* pair_buf,
                                      const LayerState& st, const CallTables& t, const CacheCallArgs& a) {
  __shared__ int s_buf_of_slot[kWave];
  __shared__ int s_any_miss, s_n_groups;
  int32_t* lds_slot_of = reinterpret_cast<int32_t*>(smem + L.slot_of);
  int32_t* lds_last = reinterpret_cast<int32_t*>(smem + L.free_buf);
  int32_t* lds_touch = reinterpret_cast<int32_t*>(smem + L.zombie);
  int32_t* lds_count = reinterpret_cast<int32_t*>(smem + L.count);
  int32_t* lds_cursor = reinterpret_cast<int32_t*>(smem + L.start);
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int C = a.C, P = a.P, K = a.K, KS = a.KS;
  const int n_lookups = a.B * K, NP = a.B * KS, NB = P + a.n_shared;
  FastTable f{};
  if (wave == 0) {
    f = fast_load(st, C, P);
    if (lane < C) s_buf_of_slot[lane] = f.buf;
    if (lane == 0) { s_any_miss = f.n_res > 0 ? 0 : 1; s_n_groups = 0; }
  }
  for (int e = tid; e < a.E; e += nthr) lds_slot_of[e] = -1;
  for (int i = tid; i < P; i += nthr) { lds_last[i] = 0; lds_touch[i] = 0; }
  for (int i = tid; i < NB; i += nthr) lds_count[i] = 0;
  __syncthreads();
  if (wave == 0 && lane < C && f.exp >= 0) lds_slot_of[f.exp] = lane;
  __syncthreads();
  {
    bool miss = false;
    for (int l = tid; l < n_lookups; l += nthr) miss |= lds_slot_of[idx[l]] < 0;
    if (miss) s_any_miss = 1;
  }
  __syncthreads();
  if (s_any_miss != 0) {                      // uniform: in-order routine, one wave
    if (wave == 0) cache_phase_fast(f, smem, L, idx, pair_buf, st, t, a);
    return;
  }
  // ---- every lookup hits ----
  const int64_t trace_n = st.scalars[SC_TRACE_N];
  for (int l = tid; l < n_lookups; l += nthr) {
    const int e = idx[l];
    const int slot = lds_slot_of[e];
    atomicMax(&lds_last[slot], l + 1);
    const int b = l / K;
    const int buf = s_buf_of_slot[slot];
    pair_buf[(size_t)b * KS + (l - b * K)] = buf;
    atomicAdd(&lds_count[buf], 1);
    if (trace_n + l < a.trace_cap) st.trace[trace_n + l] = moe_trace_rec_t{a.row0 + b, e, 1, -1};
  }
  for (int p = tid; p < a.B * a.n_shared; p += nthr) {
    const int b = p / a.n_shared, sidx = p - b * a.n_shared;
    pair_buf[(size_t)b * KS + K + sidx] = P + sidx;
    atomicAdd(&lds_count[P + sidx], 1);
  }
  __syncthreads();
  if (wave == 0) {
    // recency of the slots, buffers in use, group descriptors in ascending buffer id
    const int last = lane < C ? lds_last[lane] : 0;
    if (last > 0) {
      f.tick = (uint64_t)(f.clock + last);
      lds_touch[f.buf] = 1;
    }
    wave_sync();
    if (lane < P && lds_touch[lane]) f.used = a.seq;
    {   // buffers released by the previous call become free again (as in the in-order routine)
      const int src = lane - f.n_free;
      const int z = __shfl(f.zomb, src < 0 ? 0 : src);
      if (src >= 0 && src < f.n_zombie) f.free_b = z;
      f.n_free += f.n_zombie;
      f.n_zombie = 0;
    }
    f.clock += n_lookups;
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    int n_groups = 0, offset = 0;
    for (int base = 0; base < NB; base += kWave) {
      const int id = base + lane;
      const int c = id < NB ? lds_count[id] : 0;
      int incl = c;
#pragma unroll
      for (int dlt = 1; dlt < kWave; dlt <<= 1) {
        const int v = __shfl_up(incl, dlt);
        if (lane >= dlt) incl += v;
      }
      const int begin = offset + incl - c;
      const uint64_t gm = __ballot(c > 0);
      if (c > 0) {
        GroupDesc gd;
        gd.buf = id; gd.begin = begin; gd.count = c; gd.miss = 0;
        gd.pair0 = 0; gd.expert = -1; gd.pad[0] = gd.pad[1] = 0;
        t.grp[n_groups + __popcll(gm & lt_mask)] = gd;
      }
      if (id < NB) lds_cursor[id] = begin;
      n_groups += __popcll(gm);
      offset += __shfl(incl, kWave - 1);
    }
    if (lane == 0) { s_n_groups = n_groups; *t.n_groups = n_groups; }
    // commit the table
    if (lane < C) { st.tick[lane] = f.tick; st.expert_in[lane] = f.exp; st.buf_of_slot[lane] = f.buf; }
    if (lane < P) { st.used_stamp[lane] = f.used; st.free_buf[lane] = f.free_b; st.zombie[lane] = f.zomb; }
    if (lane == 0) {
      st.scalars[SC_CLOCK] = f.clock;
      st.scalars[SC_NRES] = f.n_res;
      st.scalars[SC_NFREE] = f.n_free;
      st.scalars[SC_NZOMBIE] = f.n_zombie;
      st.scalars[SC_CALLSEQ] = a.seq;
      st.scalars[SC_TRACE_N] = trace_n + n_lookups;
    }
  }
  __syncthreads();
  for (int p = tid; p < NP; p += nthr) {
    const int pos = atomicAdd(&lds_cursor[pair_buf[p]], 1);
    t.sorted_pair[pos] = p;
    t.pos_of[p] = pos;
  }
  __threadfence_block();
  __syncthreads();
  // a group's first pair: the smallest position belongs to whichever pair claimed it; read it back
  for (int gi = tid; gi < s_n_groups; gi += nthr) t.grp[gi].pair0 = t.sorted_pair[t.grp[gi].begin];
  if (tid == 0) {
    Mailbox* mb = a.mailbox;
    mb->status = MOE_OK;
    mb->n_miss = 0;
    mb->n_evict = 0;
    mb->n_groups = s_n_groups;
    mb->n_hits = n_lookups;
    mb->seq = a.seq;
  }
}

// Phases 1 and 2 for calls of many bf16 tokens: a workgroup (eight waves) routes a tile of 16 tokens.  The
// router logits of the tile are one small matrix product (experts x tokens) on the matrix cores: the rows of W_r
// are the A operand and the tokens the B operand of v_mfma_f32_16x16x32_bf16, both read straight from global
// memory in operand order, so W_r is read once per 16 tokens instead of once per token.  The waves then gate
// the 16 tokens between them.  The last workgroup to arrive runs phase 3 with all its waves.
__global__ void __launch_bounds__(1024) route_tile_kernel(RouteArgs r, LayerState st, CallTables t, CacheCallArgs a) {
  typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  extern __shared__ __align__(8) unsigned char smem[];
  __shared__ float zs_tile[16][kTileMaxE];
  __shared__ int s_last;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
  const int n = lane & 15, q = lane >> 4;
  const int E = a.E, K = a.K, KS = a.KS, d = r.d;
  const int t0 = blockIdx.x * 16;
  const int nkb = d >> 5;
  const uint16_t* xrow = (t0 + n < a.B) ? static_cast<const uint16_t*>(r.x) + (size_t)(t0 + n) * d + q * 8 : nullptr;
  for (int e0 = wave * 16; e0 < E; e0 += 16 * n_waves) {          // expert tiles of this wave
    const int er = e0 + n < E ? e0 + n : E - 1;         // clamped: in bounds, dropped below
    const uint16_t* wrow = static_cast<const uint16_t*>(r.router_w) + (size_t)er * d + q * 8;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    constexpr int U = 8;
    for (int kb0 = 0; kb0 < nkb; kb0 += U) {
      u32x4 wa[U], xb[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int kb = kb0 + u < nkb ? kb0 + u : nkb - 1;
        wa[u] = *reinterpret_cast<const u32x4*>(wrow + (size_t)kb * 32);
        xb[u] = xrow ? *reinterpret_cast<const u32x4*>(xrow + (size_t)kb * 32) : u32x4{0, 0, 0, 0};
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (kb0 + u < nkb)      // uniform
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wa[u]),
                                                        __builtin_bit_cast(bf16x8, xb[u]), acc, 0, 0, 0);
    }
    // lane holds experts e0 + 4q + i of token t0 + n
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = e0 + q * 4 + i;
      if (e < E && t0 + n < a.B) zs_tile[n][e] = acc[i] + (r.bias ? r.bias[(size_t)(t0 + n) * E + e] : 0.f);
    }
  }
  __syncthreads();
  for (int tt = wave; tt < 16 && t0 + tt < a.B; tt += n_waves) {
    if (E <= 64) gate_token<1>(zs_tile[tt], t0 + tt, E, K, KS, r.norm_topk, t.idx, t.wpair, r.user_idx, r.user_w, nullptr);
    else gate_token<kTileMaxE / 64>(zs_tile[tt], t0 + tt, E, K, KS, r.norm_topk, t.idx, t.wpair, r.user_idx, r.user_w,
                                    nullptr);
  }
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) s_last = atomicAdd(r.arrive, 1) == (int)gridDim.x - 1;
  __syncthreads();
  if (!s_last) return;
  if (threadIdx.x == 0) __hip_atomic_store(r.arrive, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next launch on this stream
  __threadfence();
  const LdsLayout L = lds_layout(E, a.C, a.P, a.n_shared, a.B, K, KS);
  const bool stage = stage_in_lds(a.B, KS);
  int32_t* pair_stage = stage ? reinterpret_cast<int32_t*>(smem + L.pair_stage) : t.pair_buf;
  if (a.mode == 0 && fast_table(a.policy, a.C, a.P, a.n_shared)) {
    cache_phase_fast_wide(smem, L, t.idx, pair_stage, st, t, a);
    return;
  }
  if (wave != 0) return;
  if (a.mode == 2) prefill_phase(smem, L, t.idx, pair_stage, st, t, a);
  else if (fast_table(a.policy, a.C, a.P, a.n_shared))
    cache_phase_fast(fast_load(st, a.C, a.P), smem, L, t.idx, pair_stage, st, t, a);
  else cache_phase_general(smem, L, t.idx, pair_stage, st, t, a);
}

__global__ void __launch_bounds__(64) pin_kernel(LayerState st, CallTables t, CacheCallArgs a) {
  extern __shared__ __align__(8) unsigned char smem[];
  if (fast_table(a.policy, a.C, a.P, a.n_shared)) {
    const LdsLayout L = lds_layout(a.E, a.C, a.P, a.n_shared, 1, a.K, a.KS);
    cache_phase_fast(fast_load(st, a.C, a.P), smem, L, a.pin_ids, nullptr, st, t, a);
  } else {
    const LdsLayout L = lds_layout(a.E, a.C, a.P, a.n_shared, 1, a.K, a.KS);
    cache_phase_general(smem, L, nullptr, nullptr, st, t, a);
  }
}

__global__ void reset_kernel(LayerState st, int E, int C, int P, int clear_trace, unsigned long long* dev_stats) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < C) { st.expert_in[i] = -1; st.tick[i] = 0; st.buf_of_slot[i] = -1; }
  if (i < E) st.score[i] = 0.0;
  if (i < P) { st.free_buf[i] = P - 1 - i; st.zombie[i] = -1; st.used_stamp[i] = 0; }  // buffer 0 is popped first
  if (i == 0) {
    st.scalars[SC_CLOCK] = 0;
    st.scalars[SC_NRES] = 0;
    st.scalars[SC_NFREE] = P;
    st.scalars[SC_NZOMBIE] = 0;
    if (clear_trace) st.scalars[SC_TRACE_N] = 0;
    if (dev_stats) dev_stats[0] = dev_stats[1] = dev_stats[2] = 0;
  }
}

}  // namespace

size_t route_cache_lds_bytes(int E, int C, int P, int n_shared, int B, int K, int KS) {
  return lds_layout(E, C, P, n_shared, B, K, KS).total;
}

hipError_t launch_route_cache(hipStream_t s, int dtype, const RouteArgs& r, const LayerState& st, const CallTables& t,
                              const CacheCallArgs& a, KernelEvents ev) {
  // Few tokens: 16 waves per token so that the router rows stream with many loads
  // in flight.  Many tokens: the grid supplies the parallelism.
  int waves = a.B <= 16 ? 16 : 4;
  if (waves > a.E) waves = a.E;
  dim3 grid(a.B), block(64 * waves);
  const size_t lds = route_cache_lds_bytes(a.E, a.C, a.P, a.n_shared, a.B, a.K, a.KS);
  // from about a hundred tokens on, routing 16 tokens per workgroup on the matrix cores and running the cache
  // phase on all waves of the last workgroup wins (measured: 31 against 48 us at 256 tokens, 49 against 182 us at 1024;
  // 28.6 against 26.6 at 96, 29.3 against 31.6 at 127)
  if (dtype == MOE_DTYPE_BF16 && a.B >= 112 && a.E <= kTileMaxE && r.d % 32 == 0) {
    constexpr int kTileWaves = 8;   // measured: 49 us at 1024 tokens against 61 with four waves and 54 with sixteen
    launch_timed(route_tile_kernel, dim3((a.B + 15) / 16), dim3(64 * kTileWaves), lds, s, ev, r, st, t, a);
    return hipGetLastError();
  }
  const bool one_row = a.E <= waves;
  if (dtype == MOE_DTYPE_FP32) {
    if (one_row) launch_timed(route_cache_kernel<float, 1>, grid, block, lds, s, ev, r, st, t, a);
    else launch_timed(route_cache_kernel<float, 4>, grid, block, lds, s, ev, r, st, t, a);
  } else {
    if (one_row) launch_timed(route_cache_kernel<uint16_t, 1>, grid, block, lds, s, ev, r, st, t, a);
    else launch_timed(route_cache_kernel<uint16_t, 4>, grid, block, lds, s, ev, r, st, t, a);
  }
  return hipGetLastError();
}

hipError_t launch_pin(hipStream_t s, const LayerState& st, const CallTables& t, const CacheCallArgs& a) {
  const size_t lds = route_cache_lds_bytes(a.E, a.C, a.P, a.n_shared, 1, a.K, a.KS);
  hipLaunchKernelGGL(pin_kernel, dim3(1), dim3(64), lds, s, st, t, a);
  return hipGetLastError();
}

hipError_t launch_reset(hipStream_t s, const LayerState& st, int E, int C, int P, int clear_trace,
                        unsigned long long* dev_stats) {
  int n = E > C ? E : C;
  n = n > P ? n : P;
  hipLaunchKernelGGL(reset_kernel, dim3((n + 255) / 256), dim3(256), 0, s, st, E, C, P, clear_trace, dev_stats);
  return hipGetLastError();
}

}  // namespace moe
