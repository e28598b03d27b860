// Host runtime behind the C ABI of include/moe_cache.h: owns the device expert
// buffers, the per-layer cache tables, the copy stream and the per-call
// orchestration of one MoE block (paper section 2, Eq. 1-3, under the
// offloading runtime of section 3.2).
//
// Order of one moe_layer_decode() call on the caller's stream:
//   route_cache kernel (router, gating, cache lookups, grouping; leaves the miss list and the call's counters in a
//   pinned mailbox) -> expert FFN -> combine.
// Copy-engine fetch: the FFN over the groups whose expert was already resident is enqueued before the host looks
// at the miss list; the host then reads the mailbox, issues one hipMemcpyAsync per miss (pinned pool -> device
// buffer) on the copy stream, makes the caller's stream wait for them and enqueues the FFN over the fetched
// groups.  The host round trip and the PCIe copies overlap the resident experts' compute: the additive model of
// Eq. 4 (compute + N_miss * transfer) is the worst case.
// In-kernel fetch: one FFN launch covers all groups; the workgroups of a missed expert read it from the mapped
// pinned pool and fill its device buffer on the way.  The host still reads the mailbox (counters, status) while
// that launch runs.
// A call whose evictions need more spare buffers than exist is re-issued as two waves of tokens.
#include <algorithm>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "moe_internal.hpp"
#include "q4_layout.hpp"

using namespace moe;

namespace {
thread_local char g_err[512] = "";
}

namespace moe {
int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

// Larger calls: the LDS-staged grouped GEMM (measured faster than the split-K streaming pair from 17 tokens
// on: 119 against 139 us at 17 tokens, 138 against 190 us at 128 on the OLMoE-like layer, and faster than the
// single-launch kernel from about 6 tokens: 90 against 96 us at 8, 123 against 136 us at 16).  The split-K
// pair remains for small calls on shapes the single-launch kernel does not cover.
FfnPlan plan_ffn(int pool_layout, int d, int f, int batch) {
  FfnPlan p{};
  p.tiled = pool_layout == MOE_LAYOUT_TILED;
  p.q4 = pool_layout == MOE_LAYOUT_TILED_INT4;
  p.fused = p.q4 ? batch <= 16 : (p.tiled && ffn_fused_supported(d, f, batch));
  p.gemm = p.tiled && !p.fused && batch > fused_max_tokens(f);
  return p;
}

hipError_t launch_ffn(hipStream_t s, int dtype, const FfnPlan& p, const FfnArgs& a, KernelEvents ke1, KernelEvents ke2) {
  return p.q4 ? (p.fused ? launch_ffn_fused_q4(s, a, ke1) : launch_ffn_gemm_q4(s, a, ke1, ke2))
         : p.fused ? launch_ffn_fused(s, a, ke1)
         : p.gemm ? launch_ffn_gemm(s, a, ke1, ke2)
         : p.tiled ? launch_ffn_tiled(s, a, ke1, ke2)
                   : launch_ffn_rowmajor(s, dtype, a, ke1, ke2);
}
}  // namespace moe

namespace {

#define HIPCHK(expr)                                                                        \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) return fail(MOE_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

constexpr int kProfSlots = 512;

struct ProfSlot {
  KernelEvents route, gate_up, down;   // attached to the dispatches of the three main kernels of a call
  bool used = false;
  bool tiles = false;  // ... and it was the tile kernel
  bool single = false; // the call was one launch (router to combine, timed by `gate_up`); its record is in the call log
  bool mixed = false;  // the call also fetched experts: its resident-pass FFN covers only part of the K experts
  bool fused = false;  // the call used the single-launch decode FFN (timed by `gate_up`)
  uint64_t fetched = 0; // bytes that launch read from the host pool (in-kernel fetch)
};
struct CopySlot {
  hipEvent_t c0 = nullptr, c1 = nullptr;
  uint64_t bytes = 0;
  int n = 0;
  bool used = false;
};

}  // namespace

struct moe_cache {
  moe_cache_config_t cfg{};
  moe_weights_t w{};
  int device = 0;
  int C = 0, P = 0, KS = 0, G = 0;
  uint64_t expert_bytes = 0;
  size_t elem = 2;

  char* buffers = nullptr;        // [L][P] expert blocks
  char* table_mem = nullptr;      // all LayerState arrays
  std::vector<LayerState> layers;      // [L][2]: two copies of every layer's table (see cur)
  std::vector<uint8_t> cur;            // [L] which copy is current; the single-launch decode reads it and writes the other
  unsigned long long* dev_stats = nullptr;   // [L][4] hits, misses, evictions counted on the device by calls without a host wait
  bool dev_stats_used = false;
  size_t layer_stride = 0;             // bytes between the tables (and device counters) of consecutive layers
  char* router_packed = nullptr;       // [L] router matrices in operand order, for the single-launch decode
  bool single_ok = false;              // the single-launch decode kernel covers this cache's shape and policy
  int single_max_batch = 0;
  int n_cu = 0;                        // compute units of the device
  Mailbox* call_log = nullptr;         // pinned, [kProfSlots]: call records of launches being timed
  CallTables t{};
  char* call_mem = nullptr;
  void* h = nullptr;
  float* o = nullptr;
  int32_t* arrive = nullptr;
  uint64_t wave_splits = 0;         // calls that had to be run as two waves of tokens
  std::vector<const char*> pool_host;  // [L] each layer's E expert blocks in pinned host memory
  std::vector<const char*> pool_dev;   // [L] the same as the device sees it (in-kernel fetch); empty if not mapped

  char* host_mem = nullptr;       // pinned: mailbox | pin ids | miss list
  Mailbox* mailbox = nullptr;
  int32_t* pin_ids = nullptr;
  MissEntry* miss_list = nullptr;
  int max_miss = 0;

  hipStream_t copy_stream = nullptr;
  hipEvent_t ev_mail = nullptr, ev_copy = nullptr, ev_order = nullptr;
  uint32_t seq = 0;
  bool copies_pending = false;    // copies issued that no stream has been ordered after yet

  std::vector<moe_cache_stats_t> stats;

  bool profiling = false;
  std::vector<ProfSlot> prof;
  std::vector<CopySlot> cprof;
  int prof_head = 0, cprof_head = 0;
  moe_timing_t timing{};
};

namespace {

LayerState& state_of(moe_cache* c, int layer) { return c->layers[(size_t)layer * 2 + c->cur[layer]]; }

struct DeviceGuard {
  int prev = -1;
  bool switched = false;
  hipError_t enter(int dev) {
    hipError_t e = hipGetDevice(&prev);
    if (e != hipSuccess) return e;
    if (prev != dev) {
      e = hipSetDevice(dev);
      switched = e == hipSuccess;
    }
    return e;
  }
  ~DeviceGuard() {
    if (switched) (void)hipSetDevice(prev);
  }
};

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int validate(const moe_cache_config_t* c, const moe_weights_t* w) {
  if (!c || !w) return fail(MOE_ERR_INVALID_ARG, "null config or weights");
  if (c->n_layers < 1) return fail(MOE_ERR_INVALID_ARG, "n_layers must be >= 1");
  if (c->n_experts < 1 || c->n_experts > 1024) return fail(MOE_ERR_INVALID_ARG, "n_experts must be in 1..1024");
  if (c->n_shared < 0 || c->n_shared > 64) return fail(MOE_ERR_INVALID_ARG, "n_shared must be in 0..64");
  if (c->top_k < 1 || c->top_k > c->n_experts || c->top_k > 64)
    return fail(MOE_ERR_INVALID_ARG, "top_k must be in 1..min(n_experts,64)");
  if (c->d_model < 1 || c->d_ff < 1) return fail(MOE_ERR_INVALID_ARG, "d_model and d_ff must be positive");
  if (c->dtype != MOE_DTYPE_FP32 && c->dtype != MOE_DTYPE_BF16) return fail(MOE_ERR_INVALID_ARG, "unknown dtype");
  if (c->norm_topk != 0 && c->norm_topk != 1) return fail(MOE_ERR_INVALID_ARG, "norm_topk must be 0 or 1");
  if (c->policy != MOE_POLICY_LRU && c->policy != MOE_POLICY_GAMMA) return fail(MOE_ERR_INVALID_ARG, "unknown policy");
  if (c->policy == MOE_POLICY_GAMMA && !(c->gamma >= 0.0 && c->gamma <= 1.0))
    return fail(MOE_ERR_INVALID_ARG, "gamma must be in [0,1]");
  if (c->max_batch < 1 || c->max_batch > (1 << 20)) return fail(MOE_ERR_INVALID_ARG, "max_batch out of range");
  if (c->staging_buffers < 0 || c->staging_buffers > 1024) return fail(MOE_ERR_INVALID_ARG, "staging_buffers out of range");
  if (c->trace_capacity < 0) return fail(MOE_ERR_INVALID_ARG, "trace_capacity must be >= 0");
  if (c->pool_layout != MOE_LAYOUT_ROWMAJOR && c->pool_layout != MOE_LAYOUT_TILED &&
      c->pool_layout != MOE_LAYOUT_TILED_INT4)
    return fail(MOE_ERR_INVALID_ARG, "unknown pool_layout");
  if (c->fetch_mode != MOE_FETCH_COPY_ENGINE && c->fetch_mode != MOE_FETCH_IN_KERNEL)
    return fail(MOE_ERR_INVALID_ARG, "unknown fetch_mode");
  if (c->capacity < 1) return fail(MOE_ERR_INVALID_ARG, "capacity must be >= 1");
  if (c->capacity < c->top_k)
    return fail(MOE_ERR_CAPACITY_LT_TOPK, "capacity %d < top_k %d: one token's experts would not fit", c->capacity,
                c->top_k);
  if (!w->router_w) return fail(MOE_ERR_INVALID_ARG, "router_w must not be null");
  if ((w->expert_pool != nullptr) == (w->expert_pool_layers != nullptr))
    return fail(MOE_ERR_INVALID_ARG, "exactly one of expert_pool and expert_pool_layers must be given");
  if (w->expert_pool_layers)
    for (int l = 0; l < c->n_layers; ++l)
      if (!w->expert_pool_layers[l] || (reinterpret_cast<uintptr_t>(w->expert_pool_layers[l]) & 15))
        return fail(MOE_ERR_INVALID_ARG, "expert_pool_layers[%d] is null or not 16-byte aligned", l);
  if ((c->n_shared > 0) != (w->shared_w != nullptr))
    return fail(MOE_ERR_INVALID_ARG, "shared_w must be given exactly when n_shared > 0");
  const int vec = c->dtype == MOE_DTYPE_FP32 ? 4 : 8;
  if (c->d_model % vec != 0)
    return fail(MOE_ERR_UNSUPPORTED, "d_model must be a multiple of %d for this dtype", vec);
  if (c->fetch_mode == MOE_FETCH_IN_KERNEL && (c->pool_layout == MOE_LAYOUT_ROWMAJOR || c->dtype != MOE_DTYPE_BF16))
    return fail(MOE_ERR_UNSUPPORTED, "in-kernel fetch needs a tiled layout (bf16 activations)");
  if (c->pool_layout == MOE_LAYOUT_TILED_INT4) {
    if (c->dtype != MOE_DTYPE_BF16) return fail(MOE_ERR_UNSUPPORTED, "INT4 experts need bf16 activations");
    if (!ffn_fused_q4_supported(c->d_model, c->d_ff, 1))
      return fail(MOE_ERR_UNSUPPORTED, "INT4 experts need d_model %% 256 == 0 and d_ff %% 32 == 0");
  }
  if (c->pool_layout == MOE_LAYOUT_TILED) {
    if (c->dtype != MOE_DTYPE_BF16) return fail(MOE_ERR_UNSUPPORTED, "the tiled layout is bf16 only");
    if (c->d_model % 32 != 0 || c->d_ff % 32 != 0)
      return fail(MOE_ERR_UNSUPPORTED, "the tiled layout needs d_model and d_ff to be multiples of 32");
  }
  if ((reinterpret_cast<uintptr_t>(w->router_w) & 15) || (reinterpret_cast<uintptr_t>(w->expert_pool) & 15) ||
      (reinterpret_cast<uintptr_t>(w->shared_w) & 15))
    return fail(MOE_ERR_INVALID_ARG, "weight pointers must be 16-byte aligned");
  return MOE_OK;
}

void free_all(moe_cache* c) {
  if (c->copy_stream) (void)hipStreamSynchronize(c->copy_stream);
  for (auto& p : c->prof)
    for (KernelEvents* ke : {&p.route, &p.gate_up, &p.down}) {
      if (ke->start) (void)hipEventDestroy(ke->start);
      if (ke->stop) (void)hipEventDestroy(ke->stop);
    }
  for (auto& p : c->cprof) {
    if (p.c0) (void)hipEventDestroy(p.c0);
    if (p.c1) (void)hipEventDestroy(p.c1);
  }
  if (c->ev_mail) (void)hipEventDestroy(c->ev_mail);
  if (c->ev_copy) (void)hipEventDestroy(c->ev_copy);
  if (c->ev_order) (void)hipEventDestroy(c->ev_order);
  if (c->copy_stream) (void)hipStreamDestroy(c->copy_stream);
  if (c->buffers) (void)hipFree(c->buffers);
  if (c->table_mem) (void)hipFree(c->table_mem);
  if (c->call_mem) (void)hipFree(c->call_mem);
  if (c->router_packed) (void)hipFree(c->router_packed);
  if (c->h) (void)hipFree(c->h);
  if (c->o) (void)hipFree(c->o);
  if (c->host_mem) (void)hipHostFree(c->host_mem);
  if (c->call_log) (void)hipHostFree(c->call_log);
  delete c;
}

// Wait until the cache kernel of call `seq` has filled the mailbox.
int wait_mailbox(moe_cache* c, hipStream_t s, uint32_t seq) {
  HIPCHK(hipEventRecord(c->ev_mail, s));
  HIPCHK(hipEventSynchronize(c->ev_mail));
  const uint32_t got = __atomic_load_n(&c->mailbox->seq, __ATOMIC_ACQUIRE);
  if (got != seq) return fail(MOE_ERR_TIMEOUT, "miss list of call %u not delivered (mailbox holds %u)", seq, got);
  return MOE_OK;
}

// Issue the expert copies of the current mailbox on the copy stream.
int issue_copies(moe_cache* c, int layer, int n) {
  const size_t eb = c->expert_bytes;
  const char* pool = c->pool_host[layer];
  char* bufs = c->buffers + (size_t)layer * c->P * eb;
  CopySlot* cs = nullptr;
  if (c->profiling) {
    cs = &c->cprof[c->cprof_head];
    if (cs->used) {
      HIPCHK(hipEventSynchronize(cs->c1));
      float ms = 0.f;
      HIPCHK(hipEventElapsedTime(&ms, cs->c0, cs->c1));
      c->timing.copy_ms += ms;
      c->timing.copies += cs->n;
      c->timing.copy_bytes += cs->bytes;
      cs->used = false;
    }
    HIPCHK(hipEventRecord(cs->c0, c->copy_stream));
  }
  for (int i = 0; i < n; ++i) {
    const MissEntry m = c->miss_list[i];
    if (m.expert < 0 || m.expert >= c->cfg.n_experts || m.buffer < 0 || m.buffer >= c->P)
      return fail(MOE_ERR_HIP, "corrupt miss list entry (%d,%d)", m.expert, m.buffer);
    HIPCHK(hipMemcpyAsync(bufs + (size_t)m.buffer * eb, pool + (size_t)m.expert * eb, eb, hipMemcpyHostToDevice,
                          c->copy_stream));
  }
  if (cs) {
    HIPCHK(hipEventRecord(cs->c1, c->copy_stream));
    cs->bytes = (uint64_t)n * eb;
    cs->n = n;
    cs->used = true;
    c->cprof_head = (c->cprof_head + 1) % kProfSlots;
  }
  HIPCHK(hipEventRecord(c->ev_copy, c->copy_stream));
  c->copies_pending = true;
  return MOE_OK;
}

int drain_prof_slot(moe_cache* c, ProfSlot& p) {
  if (!p.used) return MOE_OK;
  HIPCHK(hipEventSynchronize(p.fused ? p.gate_up.stop : p.down.stop));
  float a = 0.f, b = 0.f, r = 0.f;
  if (p.single) {       // one launch from the router to the combine; its call record sits in the log
    HIPCHK(hipEventElapsedTime(&a, p.gate_up.start, p.gate_up.stop));
    const Mailbox mb = c->call_log[&p - c->prof.data()];
    if (mb.n_miss > 0) {
      c->timing.fetch_launches += 1;
      c->timing.fetch_bytes += (uint64_t)mb.n_miss * c->expert_bytes;
      c->timing.fetch_ms += a;
    } else {
      c->timing.decode_single_ms += a;
      c->timing.decode_single_launches += 1;
      c->timing.decode_tiles_launches += p.tiles ? 1 : 0;
    }
    p.used = false;
    return MOE_OK;
  }
  HIPCHK(hipEventElapsedTime(&r, p.route.start, p.route.stop));
  HIPCHK(hipEventElapsedTime(&a, p.gate_up.start, p.gate_up.stop));
  if (!p.fused) HIPCHK(hipEventElapsedTime(&b, p.down.start, p.down.stop));
  c->timing.route_ms += r;
  c->timing.route_launches += 1;
  if (p.fetched) {
    c->timing.fetch_launches += 1;
    c->timing.fetch_bytes += p.fetched;
    c->timing.fetch_ms += a;
  }
  if (!p.mixed) {
    if (p.fused) {
      c->timing.ffn_fused_ms += a;
      c->timing.ffn_fused_launches += 1;
    } else {
      c->timing.ffn_gate_up_ms += a;
      c->timing.ffn_down_ms += b;
      c->timing.ffn_launches += 1;
    }
  }
  p.used = false;
  return MOE_OK;
}

}  // namespace

extern "C" {

const char* moe_last_error(void) { return g_err; }
const char* moe_version(void) { return "moe_cache 0.1 (gfx950)"; }

uint64_t moe_expert_bytes(int32_t d_model, int32_t d_ff, int32_t dtype) {
  if (d_model < 1 || d_ff < 1 || (dtype != MOE_DTYPE_FP32 && dtype != MOE_DTYPE_BF16)) return 0;
  return (uint64_t)3 * (uint64_t)d_model * (uint64_t)d_ff * (dtype == MOE_DTYPE_FP32 ? 4u : 2u);
}

uint64_t moe_expert_block_bytes(int32_t d_model, int32_t d_ff, int32_t dtype, int32_t pool_layout) {
  if (pool_layout == MOE_LAYOUT_TILED_INT4) {
    if (d_model < 128 || d_ff < 32 || d_model % 128 != 0 || d_ff % 32 != 0) return 0;
    return q4::block_bytes(d_model, d_ff);
  }
  if (pool_layout != MOE_LAYOUT_ROWMAJOR && pool_layout != MOE_LAYOUT_TILED) return 0;
  return moe_expert_bytes(d_model, d_ff, dtype);
}

int moe_pack_expert_int4(const uint8_t* codes, const uint16_t* scales, void* dst_block, int32_t d, int32_t f) {
  if (!codes || !scales || !dst_block) return fail(MOE_ERR_INVALID_ARG, "null pointer");
  if (d < 128 || f < 32 || d % 128 != 0 || f % 32 != 0)
    return fail(MOE_ERR_UNSUPPORTED, "d_model must be a positive multiple of 128 and d_ff of 32");
  for (size_t i = 0; i < (size_t)3 * d * f; ++i)
    if (codes[i] > 15) return fail(MOE_ERR_INVALID_ARG, "code %u at element %zu is not a 4-bit value", codes[i], i);
  const size_t df = (size_t)d * f;
  const uint8_t* cm[3] = {codes, codes + df, codes + 2 * df};
  const uint16_t* sm[3] = {scales, scales + df / 32, scales + 2 * (df / 32)};
  char* out = static_cast<char*>(dst_block);
  auto word = [](const uint8_t* p) {      // eight consecutive codes -> one 32-bit word
    uint32_t w = 0;
    for (int e = 0; e < 8; ++e) w |= (uint32_t)p[e] << (4 * q4::nibble_of(e));
    return w;
  };
  const int nsb = d / 128, gd = d / 32, gf = f / 32;
  for (int rt = 0; rt < f / 16; ++rt)
    for (int sb = 0; sb < nsb; ++sb) {
      char* rec = out + ((size_t)rt * nsb + sb) * q4::kGateUpRecord;
      for (int m = 0; m < 2; ++m)
        for (int l = 0; l < 64; ++l)
          for (int j = 0; j < 4; ++j) {
            const uint32_t w = word(cm[m] + (size_t)(rt * 16 + (l & 15)) * d + sb * 128 + j * 32 + (l >> 4) * 8);
            memcpy(rec + m * 1024 + l * 16 + j * 4, &w, 4);
          }
      for (int r = 0; r < 16; ++r)
        for (int m = 0; m < 2; ++m)
          memcpy(rec + 2048 + r * 16 + m * 8, sm[m] + (size_t)(rt * 16 + r) * gd + sb * 4, 8);
    }
  char* dsec = out + q4::gate_up_bytes(d, f);
  const int n_dq = d / 64;
  for (int c = 0; c < gf; ++c)
    for (int dq = 0; dq < n_dq; ++dq) {
      char* rec = dsec + ((size_t)c * n_dq + dq) * q4::kDownRecord;
      for (int l = 0; l < 64; ++l)
        for (int j = 0; j < 4; ++j) {
          const uint32_t w = word(cm[2] + (size_t)(dq * 64 + (l & 15) * 4 + j) * f + c * 32 + (l >> 4) * 8);
          memcpy(rec + l * 16 + j * 4, &w, 4);
        }
      for (int r = 0; r < 16; ++r)
        for (int j = 0; j < 4; ++j)
          memcpy(rec + 1024 + r * 8 + j * 2, sm[2] + (size_t)(dq * 64 + r * 4 + j) * gf + c, 2);
    }
  return MOE_OK;
}

int moe_pack_expert(const void* src_rowmajor, void* dst_tiled, int32_t d, int32_t f) {
  if (!src_rowmajor || !dst_tiled) return fail(MOE_ERR_INVALID_ARG, "null pointer");
  if (d < 32 || f < 32 || d % 32 != 0 || f % 32 != 0)
    return fail(MOE_ERR_UNSUPPORTED, "d_model and d_ff must be positive multiples of 32");
  const uint16_t* src = static_cast<const uint16_t*>(src_rowmajor);
  uint16_t* dst = static_cast<uint16_t*>(dst_tiled);
  const uint16_t* wg = src;
  const uint16_t* wu = src + (size_t)f * d;
  const uint16_t* wd = src + (size_t)2 * f * d;
  // gate/up section: [f/16][d/32][2][64][8]
  const int nkb_d = d / 32, nkb_f = f / 32;
  for (int ft = 0; ft < f / 16; ++ft)
    for (int kb = 0; kb < nkb_d; ++kb)
      for (int m = 0; m < 2; ++m) {
        const uint16_t* w = m == 0 ? wg : wu;
        uint16_t* out = dst + (((size_t)ft * nkb_d + kb) * 2 + m) * 512;
        for (int l = 0; l < 64; ++l)
          memcpy(out + l * 8, w + (size_t)(ft * 16 + (l & 15)) * d + kb * 32 + (l >> 4) * 8, 16);
      }
  // down section: [f/32][d/16][64][8]  (all row tiles of one 32-column block of W_d are contiguous)
  uint16_t* dsec = dst + (size_t)2 * f * d;
  for (int kb = 0; kb < nkb_f; ++kb)
    for (int dt = 0; dt < d / 16; ++dt) {
      uint16_t* out = dsec + ((size_t)kb * (d / 16) + dt) * 512;
      for (int l = 0; l < 64; ++l)
        memcpy(out + l * 8, wd + (size_t)(dt * 16 + (l & 15)) * f + kb * 32 + (l >> 4) * 8, 16);
    }
  return MOE_OK;
}

int moe_cache_create(const moe_cache_config_t* cfg, const moe_weights_t* weights, moe_cache_t** out) {
  if (out) *out = nullptr;
  if (!out) return fail(MOE_ERR_INVALID_ARG, "out must not be null");
  int rc = validate(cfg, weights);
  if (rc != MOE_OK) return rc;

  int n_dev = 0;
  hipError_t he = hipGetDeviceCount(&n_dev);
  if (he != hipSuccess || n_dev < 1) {
    (void)hipGetLastError();
    return fail(MOE_ERR_HIP, "no HIP device available (%s)", he == hipSuccess ? "device count 0" : hipGetErrorString(he));
  }
  int dev = cfg->device_id;
  if (dev < 0) HIPCHK(hipGetDevice(&dev));
  if (dev >= n_dev) return fail(MOE_ERR_INVALID_ARG, "device_id %d out of range (%d devices)", dev, n_dev);
  DeviceGuard guard;
  HIPCHK(guard.enter(dev));

  moe_cache* c = new (std::nothrow) moe_cache();
  if (!c) return fail(MOE_ERR_OUT_OF_MEMORY, "host allocation failed");
  c->cfg = *cfg;
  c->w = *weights;
  c->device = dev;
  const int L = cfg->n_layers, E = cfg->n_experts, K = cfg->top_k;
  c->C = std::min(cfg->capacity, E);
  c->P = c->C + cfg->staging_buffers;
  c->KS = K + cfg->n_shared;
  c->expert_bytes = moe_expert_block_bytes(cfg->d_model, cfg->d_ff, cfg->dtype, cfg->pool_layout);
  c->elem = cfg->dtype == MOE_DTYPE_FP32 ? 4 : 2;
  const int C = c->C, P = c->P, KS = c->KS, Bm = cfg->max_batch;
  const size_t NP = (size_t)Bm * KS;
  c->G = (int)std::min<size_t>((size_t)Bm * K, (size_t)std::max(P, E)) + cfg->n_shared;   // buffers, or experts when streaming a prompt
  c->max_miss = (int)std::max<size_t>((size_t)Bm * K, (size_t)C);
  c->stats.assign(L, moe_cache_stats_t{});

  if (route_cache_lds_bytes(E, C, P, cfg->n_shared, (int)std::min<size_t>(Bm, kStageMaxPairs / KS), K, KS) > 64 * 1024 ||
      route_cache_lds_bytes(E, C, P, cfg->n_shared, 1, C, C) > 64 * 1024) {
    delete c;
    return fail(MOE_ERR_UNSUPPORTED, "cache table of this size does not fit in LDS");
  }

#define CREATE_CHK(expr, code)                                                      \
  do {                                                                              \
    hipError_t e_ = (expr);                                                         \
    if (e_ != hipSuccess) {                                                         \
      (void)hipGetLastError();                                                      \
      free_all(c);                                                                  \
      return fail(e_ == hipErrorOutOfMemory ? MOE_ERR_OUT_OF_MEMORY : (code), "%s: %s", #expr, \
                  hipGetErrorString(e_));                                           \
    }                                                                               \
  } while (0)

  CREATE_CHK(hipMalloc(&c->buffers, (size_t)L * P * c->expert_bytes), MOE_ERR_HIP);

  // ---- per-layer tables: two copies of everything a decode call rewrites, one score array, one trace ----
  size_t ver = 0;
  const size_t o_tick = ver; ver += align_up((size_t)C * 8, 16);
  const size_t o_scal = ver; ver += align_up((size_t)SC_COUNT * 8, 16);
  const size_t o_ein = ver; ver += align_up((size_t)C * 4, 16);
  const size_t o_bos = ver; ver += align_up((size_t)C * 4, 16);
  const size_t o_free = ver; ver += align_up((size_t)P * 4, 16);
  const size_t o_zom = ver; ver += align_up((size_t)P * 4, 16);
  const size_t o_used = ver; ver += align_up((size_t)P * 4, 16);
  size_t per_layer = 2 * ver;
  const size_t o_score = per_layer; per_layer += align_up((size_t)E * 8, 16);
  const size_t o_dstat = per_layer; per_layer += 32;
  const size_t o_trace = per_layer; per_layer += align_up((size_t)cfg->trace_capacity * sizeof(moe_trace_rec_t), 16);
  CREATE_CHK(hipMalloc(&c->table_mem, per_layer * L), MOE_ERR_HIP);
  CREATE_CHK(hipMemset(c->table_mem, 0, per_layer * L), MOE_ERR_HIP);
  c->layers.resize((size_t)L * 2);
  c->cur.assign(L, 0);
  c->dev_stats = reinterpret_cast<unsigned long long*>(c->table_mem + o_dstat);   // layer l: + l * per_layer bytes
  c->layer_stride = per_layer;
  for (int l = 0; l < L; ++l)
    for (int v = 0; v < 2; ++v) {
      char* b = c->table_mem + per_layer * l;
      char* bv = b + ver * v;
      LayerState& s = c->layers[(size_t)l * 2 + v];
      s.tick = reinterpret_cast<uint64_t*>(bv + o_tick);
      s.scalars = reinterpret_cast<int64_t*>(bv + o_scal);
      s.expert_in = reinterpret_cast<int32_t*>(bv + o_ein);
      s.buf_of_slot = reinterpret_cast<int32_t*>(bv + o_bos);
      s.free_buf = reinterpret_cast<int32_t*>(bv + o_free);
      s.zombie = reinterpret_cast<int32_t*>(bv + o_zom);
      s.used_stamp = reinterpret_cast<uint32_t*>(bv + o_used);
      s.score = reinterpret_cast<double*>(b + o_score);
      s.trace = cfg->trace_capacity > 0 ? reinterpret_cast<moe_trace_rec_t*>(b + o_trace) : nullptr;
    }

  // ---- per-call scratch ----
  size_t cm = 0;
  const size_t o_idx = cm; cm += align_up((size_t)Bm * K * 4, 16);
  const size_t o_wp = cm; cm += align_up(NP * 4, 16);
  const size_t o_pb = cm; cm += align_up(NP * 4, 16);
  const size_t o_sp = cm; cm += align_up(NP * 4, 16);
  const size_t o_po = cm; cm += align_up(NP * 4, 16);
  cm = align_up(cm, 32);
  const size_t o_gd = cm; cm += (size_t)c->G * sizeof(GroupDesc);
  const size_t o_ng = cm; cm += 16;
  const size_t o_arr = cm; cm += 16;
  CREATE_CHK(hipMalloc(&c->call_mem, cm), MOE_ERR_HIP);
  CREATE_CHK(hipMemset(c->call_mem, 0, cm), MOE_ERR_HIP);
  c->t.idx = reinterpret_cast<int32_t*>(c->call_mem + o_idx);
  c->t.wpair = reinterpret_cast<float*>(c->call_mem + o_wp);
  c->t.pair_buf = reinterpret_cast<int32_t*>(c->call_mem + o_pb);
  c->t.sorted_pair = reinterpret_cast<int32_t*>(c->call_mem + o_sp);
  c->t.pos_of = reinterpret_cast<int32_t*>(c->call_mem + o_po);
  c->t.grp = reinterpret_cast<GroupDesc*>(c->call_mem + o_gd);
  c->t.n_groups = reinterpret_cast<int32_t*>(c->call_mem + o_ng);
  c->arrive = reinterpret_cast<int32_t*>(c->call_mem + o_arr);
  CREATE_CHK(hipMalloc(&c->h, NP * cfg->d_ff * 4), MOE_ERR_HIP);
  size_t o_bytes = NP * cfg->d_model * 4;
  if (cfg->pool_layout == MOE_LAYOUT_TILED_INT4 ||
      (cfg->pool_layout == MOE_LAYOUT_TILED && ffn_fused_supported(cfg->d_model, cfg->d_ff, 1))) {
    // the single-launch decode FFN keeps one partial sum per 32-row chunk of d_ff, for calls of up to 16 tokens
    const size_t pairs = (size_t)std::min(Bm, 16) * KS;
    o_bytes = std::max(o_bytes, pairs * (size_t)(cfg->d_ff / 32) * cfg->d_model * 4);
  }
  CREATE_CHK(hipMalloc(reinterpret_cast<void**>(&c->o), o_bytes), MOE_ERR_HIP);

  // ---- pinned mailbox ----
  const size_t hm = align_up(sizeof(Mailbox), 64) + align_up((size_t)C * 4, 64) + (size_t)c->max_miss * sizeof(MissEntry);
  CREATE_CHK(hipHostMalloc(reinterpret_cast<void**>(&c->host_mem), hm, hipHostMallocMapped | hipHostMallocCoherent),
             MOE_ERR_OUT_OF_MEMORY);
  memset(c->host_mem, 0, hm);
  c->mailbox = reinterpret_cast<Mailbox*>(c->host_mem);
  c->pin_ids = reinterpret_cast<int32_t*>(c->host_mem + align_up(sizeof(Mailbox), 64));
  c->miss_list = reinterpret_cast<MissEntry*>(c->host_mem + align_up(sizeof(Mailbox), 64) + align_up((size_t)C * 4, 64));

  {
    c->pool_host.resize(L);
    for (int l = 0; l < L; ++l)
      c->pool_host[l] = weights->expert_pool_layers
                            ? static_cast<const char*>(weights->expert_pool_layers[l])
                            : static_cast<const char*>(weights->expert_pool) + (size_t)l * E * c->expert_bytes;
    // the device's view of the pinned pool(s); without it only the copy engine can fetch
    std::vector<const char*> dev(L);
    bool mapped = true;
    hipError_t e_ = hipSuccess;
    if (weights->expert_pool_layers) {
      for (int l = 0; l < L && mapped; ++l) {
        void* dp = nullptr;
        e_ = hipHostGetDevicePointer(&dp, const_cast<char*>(c->pool_host[l]), 0);
        mapped = e_ == hipSuccess && dp != nullptr;
        dev[l] = static_cast<const char*>(dp);
      }
    } else {
      void* dp = nullptr;
      e_ = hipHostGetDevicePointer(&dp, const_cast<void*>(weights->expert_pool), 0);
      mapped = e_ == hipSuccess && dp != nullptr;
      for (int l = 0; l < L && mapped; ++l) dev[l] = static_cast<const char*>(dp) + (size_t)l * E * c->expert_bytes;
    }
    if (mapped) {
      c->pool_dev = dev;
    } else {
      (void)hipGetLastError();
      if (cfg->fetch_mode == MOE_FETCH_IN_KERNEL) {
        free_all(c);
        return fail(MOE_ERR_UNSUPPORTED, "in-kernel fetch: expert_pool is not device-visible pinned host memory (%s)",
                    hipGetErrorString(e_));
      }
    }
  }
  if ((cfg->pool_layout == MOE_LAYOUT_TILED || cfg->pool_layout == MOE_LAYOUT_TILED_INT4) &&
      cfg->fetch_mode == MOE_FETCH_IN_KERNEL && !c->pool_dev.empty()) {
    const int b_max = cfg->pool_layout == MOE_LAYOUT_TILED ? fused_max_tokens(cfg->d_ff) : 16;
    for (int b = 1; b <= std::min(Bm, b_max); ++b)
      if (decode_single_supported(cfg->pool_layout, cfg->policy, E, C, P, cfg->n_shared, K, cfg->d_model, cfg->d_ff, b))
        c->single_max_batch = b;
      else break;
    c->single_ok = c->single_max_batch >= 1;
  }
  CREATE_CHK(hipDeviceGetAttribute(&c->n_cu, hipDeviceAttributeMultiprocessorCount, c->device), MOE_ERR_HIP);
  if (c->single_ok) {
    CREATE_CHK(hipMalloc(&c->router_packed, router_packed_bytes(E, cfg->d_model) * L), MOE_ERR_HIP);
    CREATE_CHK(launch_pack_router(nullptr, weights->router_w, c->router_packed, E, cfg->d_model, L), MOE_ERR_HIP);
  }
  CREATE_CHK(hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking), MOE_ERR_HIP);
  CREATE_CHK(hipEventCreateWithFlags(&c->ev_mail, hipEventDisableTiming), MOE_ERR_HIP);
  CREATE_CHK(hipEventCreateWithFlags(&c->ev_copy, hipEventDisableTiming), MOE_ERR_HIP);
  CREATE_CHK(hipEventCreateWithFlags(&c->ev_order, hipEventDisableTiming), MOE_ERR_HIP);

  for (int l = 0; l < L; ++l) CREATE_CHK(launch_reset(nullptr, state_of(c, l), E, C, P, 1, nullptr), MOE_ERR_HIP);
  CREATE_CHK(hipStreamSynchronize(nullptr), MOE_ERR_HIP);
#undef CREATE_CHK
  *out = c;
  return MOE_OK;
}

int moe_cache_destroy(moe_cache_t* c) {
  if (!c) return MOE_OK;
  DeviceGuard guard;
  HIPCHK(guard.enter(c->device));
  (void)hipDeviceSynchronize();
  free_all(c);
  return MOE_OK;
}

int moe_cache_reset(moe_cache_t* c, int32_t layer, int32_t clear_stats, void* hip_stream) {
  if (!c) return fail(MOE_ERR_INVALID_ARG, "null cache");
  if (layer < -1 || layer >= c->cfg.n_layers) return fail(MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
  DeviceGuard guard;
  HIPCHK(guard.enter(c->device));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int l0 = layer < 0 ? 0 : layer, l1 = layer < 0 ? c->cfg.n_layers : layer + 1;
  for (int l = l0; l < l1; ++l) {
    unsigned long long* ds = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(c->dev_stats) + c->layer_stride * l);
    HIPCHK(launch_reset(s, state_of(c, l), c->cfg.n_experts, c->C, c->P, clear_stats ? 1 : 0, clear_stats ? ds : nullptr));
    if (clear_stats) c->stats[l] = moe_cache_stats_t{};
  }
  return MOE_OK;
}

int moe_cache_prefill_pins(moe_cache_t* c, int32_t layer, const int32_t* expert_ids, int32_t n, void* hip_stream) {
  if (!c) return fail(MOE_ERR_INVALID_ARG, "null cache");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
  if (n < 0 || n > c->C) return fail(MOE_ERR_INVALID_ARG, "n = %d pins exceed the capacity %d", n, c->C);
  if (n == 0) return MOE_OK;
  if (!expert_ids) return fail(MOE_ERR_INVALID_ARG, "expert_ids must not be null");
  for (int i = 0; i < n; ++i) {
    if (expert_ids[i] < 0 || expert_ids[i] >= c->cfg.n_experts)
      return fail(MOE_ERR_INVALID_ARG, "pin id %d out of range", expert_ids[i]);
    for (int j = 0; j < i; ++j)
      if (expert_ids[j] == expert_ids[i]) return fail(MOE_ERR_INVALID_ARG, "duplicate pin id %d", expert_ids[i]);
  }
  DeviceGuard guard;
  HIPCHK(guard.enter(c->device));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  memcpy(c->pin_ids, expert_ids, (size_t)n * 4);

  CacheCallArgs a{};
  a.mode = 1; a.B = 1; a.K = n; a.KS = n; a.E = c->cfg.n_experts; a.C = c->C; a.P = c->P;
  a.n_shared = c->cfg.n_shared; a.policy = c->cfg.policy; a.gamma = c->cfg.gamma;
  a.trace_cap = c->cfg.trace_capacity; a.seq = ++c->seq; a.pin_ids = c->pin_ids;
  a.mailbox = c->mailbox; a.miss_list = c->miss_list; a.max_miss = c->max_miss;
  if (c->copies_pending) { HIPCHK(hipStreamWaitEvent(s, c->ev_copy, 0)); c->copies_pending = false; }
  HIPCHK(launch_pin(s, state_of(c, layer), c->t, a));
  int rc = wait_mailbox(c, s, a.seq);
  if (rc != MOE_OK) return rc;
  const Mailbox mb = *c->mailbox;
  if (mb.status != MOE_OK) return fail(mb.status, "prefill_pins ran out of expert buffers");
  if (mb.n_miss > 0) {
    rc = issue_copies(c, layer, mb.n_miss);
    if (rc != MOE_OK) return rc;
    HIPCHK(hipStreamWaitEvent(s, c->ev_copy, 0));
    c->copies_pending = false;
  }
  moe_cache_stats_t& st = c->stats[layer];
  st.pin_loads += (uint64_t)mb.n_miss;
  st.evictions += (uint64_t)mb.n_evict;
  st.bytes_h2d += (uint64_t)mb.n_miss * c->expert_bytes;
  return MOE_OK;
}

}  // extern "C"

namespace {

// One wave of tokens: the whole call when its evictions fit the spare buffers.
int decode_wave(moe_cache_t* c, int32_t layer, const void* x_dev, const float* logit_bias_dev, int32_t batch,
                void* y_dev, int32_t* topk_idx_dev, float* topk_w_dev, hipStream_t s, int32_t row0) {
  const moe_cache_config_t& cf = c->cfg;
  const int E = cf.n_experts, K = cf.top_k, KS = c->KS, d = cf.d_model;

  ProfSlot* ps = nullptr;
  if (c->profiling) {
    ps = &c->prof[c->prof_head];
    int rc = drain_prof_slot(c, *ps);
    if (rc != MOE_OK) return rc;
    c->prof_head = (c->prof_head + 1) % kProfSlots;
  }

  RouteArgs ra{};
  ra.x = x_dev;
  ra.router_w = static_cast<const char*>(c->w.router_w) + (size_t)layer * E * d * c->elem;
  ra.bias = logit_bias_dev;
  ra.d = d; ra.norm_topk = cf.norm_topk;
  ra.user_idx = topk_idx_dev; ra.user_w = topk_w_dev;
  ra.arrive = c->arrive;

  // One launch up to the combine, and no host wait: batch 1 (a single token's experts always fit), or a cache
  // that holds every expert (nothing is ever evicted) - the two cases in which a call cannot run out of spare
  // buffers - on the shapes the single-launch kernel covers.
  if (c->single_ok && batch <= c->single_max_batch && (batch == 1 || c->C >= E)) {
    RoutedArgs q{};
    q.r = ra;
    q.router_packed = c->router_packed + router_packed_bytes(E, d) * layer;
    q.st_in = state_of(c, layer);
    q.st_out = c->layers[(size_t)layer * 2 + (c->cur[layer] ^ 1)];
    CacheCallArgs& a = q.a;
    a.mode = 0; a.B = batch; a.K = K; a.KS = KS; a.E = E; a.C = c->C; a.P = c->P; a.n_shared = cf.n_shared;
    a.row0 = row0;
    a.policy = cf.policy; a.gamma = cf.gamma; a.trace_cap = cf.trace_capacity; a.seq = ++c->seq;
    a.pin_ids = nullptr; a.mailbox = c->mailbox; a.miss_list = c->miss_list; a.max_miss = c->max_miss;
    q.dev_stats = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(c->dev_stats) + c->layer_stride * layer);
    q.log = ps ? c->call_log + (ps - c->prof.data()) : nullptr;
    FfnArgs fa{};
    fa.x = x_dev;
    fa.buffers = c->buffers + (size_t)layer * c->P * c->expert_bytes;
    fa.shared = cf.n_shared ? static_cast<const char*>(c->w.shared_w) + (size_t)layer * cf.n_shared * c->expert_bytes
                            : nullptr;
    fa.expert_bytes = c->expert_bytes;
    fa.P = c->P; fa.d = d; fa.f = cf.d_ff; fa.KS = KS;
    fa.g_max = (int)std::min<size_t>((size_t)batch * K, (size_t)c->P) + cf.n_shared;
    fa.max_count = batch;
    fa.t = c->t; fa.h = c->h; fa.o = c->o;
    fa.fused = 1; fa.pass = 2;
    fa.pool = c->pool_dev[layer];
    fa.fetch = 1;
    fa.n_parts = decode_tiles_parts(cf.pool_layout, d, cf.d_ff, batch, fa.g_max, c->n_cu, E);
    if (fa.n_parts > 0) HIPCHK(launch_decode_tiles(s, fa, q, ps ? ps->gate_up : KernelEvents{}));
    else HIPCHK(launch_decode_single(s, cf.pool_layout, fa, q, ps ? ps->gate_up : KernelEvents{}));
    HIPCHK(launch_combine_chunks(s, c->o, c->t.wpair, c->t.pos_of, batch, KS, d,
                                 fa.n_parts > 0 ? fa.n_parts : cf.d_ff / 32, y_dev, batch == 1));
    c->cur[layer] ^= 1;
    c->dev_stats_used = true;
    c->stats[layer].lookups += (uint64_t)batch * K;
    if (ps) { ps->used = true; ps->single = true; ps->tiles = fa.n_parts > 0; ps->fused = true; ps->mixed = false; ps->fetched = 0; }
    return MOE_OK;
  }

  CacheCallArgs a{};
  a.mode = 0; a.B = batch; a.K = K; a.KS = KS; a.E = E; a.C = c->C; a.P = c->P; a.n_shared = cf.n_shared;
  a.row0 = row0;
  a.policy = cf.policy; a.gamma = cf.gamma; a.trace_cap = cf.trace_capacity; a.seq = ++c->seq;
  a.pin_ids = nullptr; a.mailbox = c->mailbox; a.miss_list = c->miss_list; a.max_miss = c->max_miss;
  HIPCHK(launch_route_cache(s, cf.dtype, ra, state_of(c, layer), c->t, a, ps ? ps->route : KernelEvents{}));
  HIPCHK(hipEventRecord(c->ev_mail, s));

  FfnArgs fa{};
  fa.x = x_dev;
  fa.buffers = c->buffers + (size_t)layer * c->P * c->expert_bytes;
  fa.shared = cf.n_shared ? static_cast<const char*>(c->w.shared_w) + (size_t)layer * cf.n_shared * c->expert_bytes
                          : nullptr;
  fa.expert_bytes = c->expert_bytes;
  fa.P = c->P; fa.d = d; fa.f = cf.d_ff; fa.KS = KS;
  fa.g_max = (int)std::min<size_t>((size_t)batch * K, (size_t)c->P) + cf.n_shared;
  fa.max_count = batch;
  fa.t = c->t; fa.h = c->h; fa.o = c->o;
  const FfnPlan plan = plan_ffn(cf.pool_layout, d, cf.d_ff, batch);
  const bool fused = plan.fused;
  fa.fused = fused ? 1 : 0;
  const KernelEvents ke1 = ps ? ps->gate_up : KernelEvents{}, ke2 = ps ? ps->down : KernelEvents{};

  // Experts that were already resident: their FFN starts right behind the cache
  // lookups, before the host knows the miss list.  With in-kernel fetch the same
  // launch also streams the missed experts from the host pool.
  const bool in_kernel = fused && cf.fetch_mode == MOE_FETCH_IN_KERNEL;
  fa.pool = in_kernel ? c->pool_dev[layer] : nullptr;
  fa.fetch = in_kernel ? 1 : 0;
  fa.pass = in_kernel ? 2 : 0;
  HIPCHK(launch_ffn(s, cf.dtype, plan, fa, ke1, ke2));

  HIPCHK(hipEventSynchronize(c->ev_mail));
  const uint32_t got = __atomic_load_n(&c->mailbox->seq, __ATOMIC_ACQUIRE);
  if (got != a.seq) return fail(MOE_ERR_TIMEOUT, "miss list of call %u not delivered (mailbox holds %u)", a.seq, got);
  const Mailbox mb = *c->mailbox;
  if (mb.status != MOE_OK)
    return fail(mb.status, "call needs more spare expert buffers than staging_buffers=%d (batch %d)",
                cf.staging_buffers, batch);
  if (mb.n_miss > 0 && !in_kernel) {
    int rc = issue_copies(c, layer, mb.n_miss);
    if (rc != MOE_OK) return rc;
    HIPCHK(hipStreamWaitEvent(s, c->ev_copy, 0));
    c->copies_pending = false;
    fa.pass = 1;
    HIPCHK(launch_ffn(s, cf.dtype, plan, fa, KernelEvents{}, KernelEvents{}));
  }
  if (ps) {
    ps->used = true; ps->single = false; ps->mixed = mb.n_miss > 0; ps->fused = fused;
    ps->fetched = in_kernel ? (uint64_t)mb.n_miss * c->expert_bytes : 0;
  }
  HIPCHK(fused ? launch_combine_chunks(s, c->o, c->t.wpair, c->t.pos_of, batch, KS, d, cf.d_ff / 32, y_dev)
               : launch_combine(s, cf.dtype, c->o, c->t.wpair, c->t.pos_of, batch, KS, d, y_dev));

  moe_cache_stats_t& st = c->stats[layer];
  st.lookups += (uint64_t)batch * K;
  st.hits += (uint64_t)mb.n_hits;
  st.misses += (uint64_t)mb.n_miss;
  st.evictions += (uint64_t)mb.n_evict;
  st.bytes_h2d += (uint64_t)mb.n_miss * c->expert_bytes;
  return MOE_OK;
}

// A call whose evictions need more spare buffers than exist changes nothing on the device; it is then run as two
// consecutive waves of tokens (recursively).  Tokens are looked up in row order either way, so hits, misses,
// evictions and outputs are those of the unsplit call.  A single token always fits (K <= C).
int decode_rows(moe_cache_t* c, int32_t layer, const char* x, const float* bias, int32_t batch, char* y,
                int32_t* idx, float* w, hipStream_t s, int32_t row0) {
  const int rc = decode_wave(c, layer, x, bias, batch, y, idx, w, s, row0);
  if (rc != MOE_ERR_STAGING_EXHAUSTED || batch == 1) return rc;
  ++c->wave_splits;
  const int n1 = batch / 2;
  const size_t row = (size_t)c->cfg.d_model * c->elem;
  const int E = c->cfg.n_experts, K = c->cfg.top_k;
  const int rc1 = decode_rows(c, layer, x, bias, n1, y, idx, w, s, row0);
  if (rc1 != MOE_OK) return rc1;
  return decode_rows(c, layer, x + n1 * row, bias ? bias + (size_t)n1 * E : nullptr, batch - n1, y + n1 * row,
                     idx ? idx + (size_t)n1 * K : nullptr, w ? w + (size_t)n1 * K : nullptr, s, row0 + n1);
}

}  // namespace

extern "C" {

int moe_layer_decode(moe_cache_t* c, int32_t layer, const void* x_dev, const float* logit_bias_dev, int32_t batch,
                     void* y_dev, int32_t* topk_idx_dev, float* topk_w_dev, void* hip_stream) {
  if (!c) return fail(MOE_ERR_INVALID_ARG, "null cache");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
  if (!x_dev || !y_dev) return fail(MOE_ERR_INVALID_ARG, "x_dev and y_dev must not be null");
  if (batch < 1 || batch > c->cfg.max_batch)
    return fail(MOE_ERR_INVALID_ARG, "batch %d outside 1..max_batch=%d", batch, c->cfg.max_batch);
  if (reinterpret_cast<uintptr_t>(x_dev) & 15) return fail(MOE_ERR_INVALID_ARG, "x_dev must be 16-byte aligned");
  DeviceGuard guard;
  HIPCHK(guard.enter(c->device));
  return decode_rows(c, layer, static_cast<const char*>(x_dev), logit_bias_dev, batch, static_cast<char*>(y_dev),
                     topk_idx_dev, topk_w_dev, static_cast<hipStream_t>(hip_stream), 0);
}

int moe_pooled_prefetch_set(const float* scores, int32_t n_seqs, int32_t n_experts, int32_t capacity,
                            int32_t* ids_out, int32_t* n_out) {
  if (!scores || !ids_out || !n_out) return fail(MOE_ERR_INVALID_ARG, "null pointer");
  if (n_seqs < 1 || n_experts < 1 || capacity < 1) return fail(MOE_ERR_INVALID_ARG, "sizes must be positive");
  std::vector<double> total((size_t)n_experts, 0.0);
  for (int sq = 0; sq < n_seqs; ++sq)
    for (int e = 0; e < n_experts; ++e) total[e] += (double)scores[(size_t)sq * n_experts + e];
  std::vector<int32_t> order((size_t)n_experts);
  for (int e = 0; e < n_experts; ++e) order[e] = e;
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return total[a] > total[b]; });
  const int n = std::min(capacity, n_experts);
  for (int i = 0; i < n; ++i) ids_out[i] = order[n - 1 - i];     // best score last = most recently used
  *n_out = n;
  return MOE_OK;
}

int moe_layer_prefill(moe_cache_t* c, int32_t layer, const void* x_dev, const float* logit_bias_dev, int32_t n_tokens,
                      void* y_dev, int32_t* topk_idx_dev, float* topk_w_dev, void* hip_stream) {
  if (!c) return fail(MOE_ERR_INVALID_ARG, "null cache");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
  if (!x_dev || !y_dev) return fail(MOE_ERR_INVALID_ARG, "x_dev and y_dev must not be null");
  if (n_tokens < 1 || n_tokens > c->cfg.max_batch)
    return fail(MOE_ERR_INVALID_ARG, "n_tokens %d outside 1..max_batch=%d", n_tokens, c->cfg.max_batch);
  if (reinterpret_cast<uintptr_t>(x_dev) & 15) return fail(MOE_ERR_INVALID_ARG, "x_dev must be 16-byte aligned");
  if (c->cfg.pool_layout == MOE_LAYOUT_ROWMAJOR) return fail(MOE_ERR_UNSUPPORTED, "prompt streaming needs a tiled layout");
  if (c->pool_dev.empty()) return fail(MOE_ERR_UNSUPPORTED, "prompt streaming: expert_pool is not device-visible pinned host memory");
  DeviceGuard guard;
  HIPCHK(guard.enter(c->device));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const moe_cache_config_t& cf = c->cfg;
  const int E = cf.n_experts, K = cf.top_k, KS = c->KS, d = cf.d_model;

  RouteArgs ra{};
  ra.x = x_dev;
  ra.router_w = static_cast<const char*>(c->w.router_w) + (size_t)layer * E * d * c->elem;
  ra.bias = logit_bias_dev;
  ra.d = d; ra.norm_topk = cf.norm_topk;
  ra.user_idx = topk_idx_dev; ra.user_w = topk_w_dev;
  ra.arrive = c->arrive;

  CacheCallArgs a{};
  a.mode = 2; a.B = n_tokens; a.K = K; a.KS = KS; a.E = E; a.C = c->C; a.P = c->P; a.n_shared = cf.n_shared;
  a.policy = cf.policy; a.gamma = cf.gamma; a.trace_cap = 0; a.seq = ++c->seq;
  a.pin_ids = nullptr; a.mailbox = c->mailbox; a.miss_list = c->miss_list; a.max_miss = c->max_miss;
  HIPCHK(launch_route_cache(s, cf.dtype, ra, state_of(c, layer), c->t, a, KernelEvents{}));
  HIPCHK(hipEventRecord(c->ev_mail, s));

  FfnArgs fa{};
  fa.x = x_dev;
  fa.buffers = c->buffers + (size_t)layer * c->P * c->expert_bytes;
  fa.shared = cf.n_shared ? static_cast<const char*>(c->w.shared_w) + (size_t)layer * cf.n_shared * c->expert_bytes
                          : nullptr;
  fa.expert_bytes = c->expert_bytes;
  fa.P = c->P; fa.d = d; fa.f = cf.d_ff; fa.KS = KS;
  fa.g_max = (int)std::min<size_t>((size_t)n_tokens * K, (size_t)E) + cf.n_shared;   // groups are experts here
  fa.max_count = n_tokens;
  fa.t = c->t; fa.h = c->h; fa.o = c->o;
  fa.pass = 2; fa.fused = 0;
  fa.pool = c->pool_dev[layer];
  fa.fetch = 1;
  HIPCHK(cf.pool_layout == MOE_LAYOUT_TILED_INT4 ? launch_ffn_gemm_q4(s, fa, KernelEvents{}, KernelEvents{})
                                                  : launch_ffn_gemm(s, fa, KernelEvents{}, KernelEvents{}));

  HIPCHK(hipEventSynchronize(c->ev_mail));
  const uint32_t got = __atomic_load_n(&c->mailbox->seq, __ATOMIC_ACQUIRE);
  if (got != a.seq) return fail(MOE_ERR_TIMEOUT, "group list of call %u not delivered (mailbox holds %u)", a.seq, got);
  const Mailbox mb = *c->mailbox;
  HIPCHK(launch_combine(s, cf.dtype, c->o, c->t.wpair, c->t.pos_of, n_tokens, KS, d, y_dev));
  moe_cache_stats_t& st = c->stats[layer];
  st.stream_loads += (uint64_t)mb.n_miss;
  st.bytes_streamed += (uint64_t)mb.n_miss * c->expert_bytes;
  return MOE_OK;
}

int moe_cache_stats(const moe_cache_t* c, int32_t layer, moe_cache_stats_t* out) {
  if (!c || !out) return fail(MOE_ERR_INVALID_ARG, "null argument");
  if (layer < -1 || layer >= c->cfg.n_layers) return fail(MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
  const int L = c->cfg.n_layers;
  // calls that did not wait for the device counted their hits, misses and evictions there
  std::vector<unsigned long long> dev((size_t)L * 4, 0ull);
  if (c->dev_stats_used) {
    DeviceGuard guard;
    HIPCHK(guard.enter(c->device));
    HIPCHK(hipDeviceSynchronize());
    HIPCHK(hipMemcpy2D(dev.data(), 32, c->dev_stats, c->layer_stride, 32, L, hipMemcpyDeviceToHost));
  }
  moe_cache_stats_t s{};
  const int l0 = layer < 0 ? 0 : layer, l1 = layer < 0 ? L : layer + 1;
  for (int l = l0; l < l1; ++l) {
    const moe_cache_stats_t& v = c->stats[l];
    const unsigned long long* dv = &dev[(size_t)l * 4];
    s.lookups += v.lookups; s.hits += v.hits + dv[0]; s.misses += v.misses + dv[1];
    s.evictions += v.evictions + dv[2]; s.pin_loads += v.pin_loads;
    s.bytes_h2d += v.bytes_h2d + dv[1] * c->expert_bytes;
    s.stream_loads += v.stream_loads; s.bytes_streamed += v.bytes_streamed;
  }
  *out = s;
  return MOE_OK;
}

int moe_cache_read_trace(moe_cache_t* c, int32_t layer, moe_trace_rec_t* host_out, int64_t max_records,
                         int64_t* n_out, int64_t* n_total) {
  if (!c || !n_out) return fail(MOE_ERR_INVALID_ARG, "null argument");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
  if (max_records < 0 || (max_records > 0 && !host_out)) return fail(MOE_ERR_INVALID_ARG, "bad output buffer");
  DeviceGuard guard;
  HIPCHK(guard.enter(c->device));
  HIPCHK(hipDeviceSynchronize());
  int64_t total = 0;
  HIPCHK(hipMemcpy(&total, state_of(c, layer).scalars + SC_TRACE_N, 8, hipMemcpyDeviceToHost));
  int64_t n = std::min<int64_t>(std::min<int64_t>(total, c->cfg.trace_capacity), max_records);
  if (n > 0) HIPCHK(hipMemcpy(host_out, state_of(c, layer).trace, (size_t)n * sizeof(moe_trace_rec_t), hipMemcpyDeviceToHost));
  *n_out = n;
  if (n_total) *n_total = total;
  return MOE_OK;
}

int moe_cache_resident(moe_cache_t* c, int32_t layer, int32_t* host_out, int32_t* n_out) {
  if (!c || !host_out || !n_out) return fail(MOE_ERR_INVALID_ARG, "null argument");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(MOE_ERR_INVALID_ARG, "layer %d out of range", layer);
  DeviceGuard guard;
  HIPCHK(guard.enter(c->device));
  HIPCHK(hipDeviceSynchronize());
  std::vector<int32_t> ein(c->C);
  HIPCHK(hipMemcpy(ein.data(), state_of(c, layer).expert_in, (size_t)c->C * 4, hipMemcpyDeviceToHost));
  std::vector<int32_t> res;
  for (int v : ein) if (v >= 0) res.push_back(v);
  std::sort(res.begin(), res.end());
  for (size_t i = 0; i < res.size(); ++i) host_out[i] = res[i];
  *n_out = (int32_t)res.size();
  return MOE_OK;
}

int moe_cache_set_profiling(moe_cache_t* c, int32_t enabled) {
  if (!c) return fail(MOE_ERR_INVALID_ARG, "null cache");
  DeviceGuard guard;
  HIPCHK(guard.enter(c->device));
  if (enabled && c->prof.empty()) {
    c->prof.resize(kProfSlots);
    c->cprof.resize(kProfSlots);
    for (auto& p : c->prof)
      for (KernelEvents* ke : {&p.route, &p.gate_up, &p.down}) {
        HIPCHK(hipEventCreate(&ke->start));
        HIPCHK(hipEventCreate(&ke->stop));
      }
    for (auto& p : c->cprof) { HIPCHK(hipEventCreate(&p.c0)); HIPCHK(hipEventCreate(&p.c1)); }
    HIPCHK(hipHostMalloc(reinterpret_cast<void**>(&c->call_log), kProfSlots * sizeof(Mailbox),
                         hipHostMallocMapped | hipHostMallocCoherent));
    memset(c->call_log, 0, kProfSlots * sizeof(Mailbox));
  }
  c->profiling = enabled != 0;
  return MOE_OK;
}

int moe_cache_timing(moe_cache_t* c, moe_timing_t* out, int32_t clear) {
  if (!c || !out) return fail(MOE_ERR_INVALID_ARG, "null argument");
  DeviceGuard guard;
  HIPCHK(guard.enter(c->device));
  for (auto& p : c->prof) {
    int rc = drain_prof_slot(c, p);
    if (rc != MOE_OK) return rc;
  }
  for (auto& cs : c->cprof) {
    if (!cs.used) continue;
    HIPCHK(hipEventSynchronize(cs.c1));
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, cs.c0, cs.c1));
    c->timing.copy_ms += ms;
    c->timing.copies += cs.n;
    c->timing.copy_bytes += cs.bytes;
    cs.used = false;
  }
  *out = c->timing;
  if (clear) c->timing = moe_timing_t{};
  return MOE_OK;
}

}  // extern "C"
