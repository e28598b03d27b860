// Device-resident expert-cache table: lookup, eviction, buffer assignment and
// the token -> expert grouping of one MoE layer call.
//
// Follows the offloading runtime of paper section 2 ("Expert Offloading
// Systems") and section 3.2: a selected expert that is not resident is fetched
// on demand and a cached expert is evicted as the policy dictates.  LRU is the
// gamma -> 0+ member and LFU the gamma = 1 member of the discounted-count
// family of Definition C.1; contents change lazily, only by inserting the
// requested expert (Remark after Definition C.1).
//
// One wavefront runs the whole call: lookups are inherently sequential (each
// one changes the state the next one sees), so the table lives in LDS for the
// duration of the kernel and only the victim search and the table load/store
// are spread over the lanes.  Nothing is committed to global memory when the
// call runs out of spare buffers, so a failed call leaves the cache unchanged.
#include "device_utils.hpp"
#include "moe_internal.hpp"

namespace moe {

namespace {

struct LdsLayout {
  size_t tick, score, expert_in, buf_of_slot, slot_of, free_buf, zombie, used, filled, pending, count, start, total;
};

__host__ __device__ inline LdsLayout lds_layout(int E, int C, int P, int n_shared) {
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
  l.count = o; o += (size_t)(P + n_shared) * 4;
  l.start = o; o += (size_t)(P + n_shared) * 4;
  l.total = o;
  return l;
}

}  // namespace

size_t cache_kernel_lds_bytes(const CacheCallArgs& a) { return lds_layout(a.E, a.C, a.P, a.n_shared).total; }

__global__ void __launch_bounds__(64) cache_kernel(LayerState st, CallTables t, CacheCallArgs a) {
  extern __shared__ __align__(8) unsigned char smem[];
  const LdsLayout L = lds_layout(a.E, a.C, a.P, a.n_shared);
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

  const int lane = threadIdx.x;
  const int E = a.E, C = a.C, P = a.P, K = a.K, KS = a.KS;
  const bool gamma_policy = a.policy == MOE_POLICY_GAMMA;

  // ---- load the table ----
  for (int s = lane; s < C; s += kWave) {
    tick[s] = st.tick[s]; expert_in[s] = st.expert_in[s]; buf_of_slot[s] = st.buf_of_slot[s];
  }
  for (int e = lane; e < E; e += kWave) {
    slot_of[e] = st.slot_of[e]; pending[e] = 0;
    if (gamma_policy) score[e] = st.score[e];
  }
  int64_t clock = st.scalars[SC_CLOCK];
  int n_res = (int)st.scalars[SC_NRES];
  int n_free = (int)st.scalars[SC_NFREE];
  int n_zombie = (int)st.scalars[SC_NZOMBIE];
  int64_t trace_n = st.scalars[SC_TRACE_N];
  for (int i = lane; i < n_free; i += kWave) free_buf[i] = st.free_buf[i];
  // buffers released by the previous call: all its kernels have finished, reuse them
  for (int i = lane; i < n_zombie; i += kWave) free_buf[n_free + i] = st.zombie[i];
  n_free += n_zombie;
  n_zombie = 0;
  for (int i = lane; i < P; i += kWave) { used[i] = st.used_stamp[i]; filled[i] = 0; }
  __syncthreads();

  const uint32_t seq = a.seq;
  const int n_lookups = a.mode == 0 ? a.B * K : K;
  int status = MOE_OK, n_miss = 0, n_evict = 0, n_hits = 0;
  int64_t trace_added = 0;

  for (int q = 0; q < n_lookups; ++q) {
    const int b = a.mode == 0 ? q / K : 0;
    const int k = a.mode == 0 ? q % K : q;
    const int e = a.mode == 0 ? t.idx[q] : a.pin_ids[q];
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
        filled[buf] = 1;
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
        t.pair_buf[(size_t)b * KS + k] = buf;
        if (trace_n + trace_added < a.trace_cap)
          st.trace[trace_n + trace_added] = moe_trace_rec_t{b, e, hit ? 1 : 0, evicted};
      }
    }
    if (a.mode == 0) ++trace_added;
    __syncthreads();
    // Definition C.1: the discounted counts advance once per token (each pinned expert is a token)
    if (a.mode == 1 || k == K - 1) {
      if (gamma_policy) {
        for (int x = lane; x < E; x += kWave)
          score[x] = __dadd_rn(__dmul_rn(a.gamma, score[x]), (double)pending[x]);
      }
      for (int x = lane; x < E; x += kWave) pending[x] = 0;
      __syncthreads();
    }
  }

  int n_groups = 0;
  if (status == MOE_OK && a.mode == 0) {
    // ---- group the (token, expert) pairs by the buffer they read: stable counting sort ----
    const int NP = a.B * KS;
    const int NB = P + a.n_shared;
    for (int p = lane; p < a.B * a.n_shared; p += kWave) {
      const int b = p / a.n_shared, sidx = p % a.n_shared;
      t.pair_buf[(size_t)b * KS + K + sidx] = P + sidx;
    }
    for (int i = lane; i < NB; i += kWave) count[i] = 0;
    __syncthreads();
    for (int p = lane; p < NP; p += kWave) atomicAdd(&count[t.pair_buf[p]], 1);
    __syncthreads();
    if (lane == 0) {
      int off = 0;
      for (int id = 0; id < NB; ++id) {
        const int c = count[id];
        if (c > 0) {
          t.grp_buf[n_groups] = id;
          t.grp_begin[n_groups] = off;
          t.grp_count[n_groups] = c;
          t.grp_miss[n_groups] = id < P ? filled[id] : 0;
          ++n_groups;
        }
        start[id] = off;
        off += c;
      }
      for (int p = 0; p < NP; ++p) {
        const int pos = start[t.pair_buf[p]]++;
        t.sorted_pair[pos] = p;
        t.pos_of[p] = pos;
      }
    }
    n_groups = __shfl(n_groups, 0);
  }
  if (a.mode == 0 && lane == 0) *t.n_groups = n_groups;

  if (status == MOE_OK) {
    // ---- commit ----
    __syncthreads();
    for (int s = lane; s < C; s += kWave) {
      st.tick[s] = tick[s]; st.expert_in[s] = expert_in[s]; st.buf_of_slot[s] = buf_of_slot[s];
    }
    for (int e = lane; e < E; e += kWave) {
      st.slot_of[e] = slot_of[e];
      if (gamma_policy) st.score[e] = score[e];
    }
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
    __threadfence_system();
    __hip_atomic_store(&mb->seq, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
  }
}

__global__ void reset_kernel(LayerState st, int E, int C, int P, int clear_trace) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < C) { st.expert_in[i] = -1; st.tick[i] = 0; st.buf_of_slot[i] = -1; }
  if (i < E) { st.slot_of[i] = -1; st.score[i] = 0.0; }
  if (i < P) { st.free_buf[i] = P - 1 - i; st.zombie[i] = -1; st.used_stamp[i] = 0; }  // buffer 0 is popped first
  if (i == 0) {
    st.scalars[SC_CLOCK] = 0;
    st.scalars[SC_NRES] = 0;
    st.scalars[SC_NFREE] = P;
    st.scalars[SC_NZOMBIE] = 0;
    if (clear_trace) st.scalars[SC_TRACE_N] = 0;
  }
}

hipError_t launch_cache(hipStream_t s, const LayerState& st, const CallTables& t, const CacheCallArgs& a) {
  hipLaunchKernelGGL(cache_kernel, dim3(1), dim3(64), cache_kernel_lds_bytes(a), s, st, t, a);
  return hipGetLastError();
}

hipError_t launch_reset(hipStream_t s, const LayerState& st, int E, int C, int P, int clear_trace) {
  int n = E > C ? E : C;
  n = n > P ? n : P;
  hipLaunchKernelGGL(reset_kernel, dim3((n + 255) / 256), dim3(256), 0, s, st, E, C, P, clear_trace);
  return hipGetLastError();
}

}  // namespace moe
