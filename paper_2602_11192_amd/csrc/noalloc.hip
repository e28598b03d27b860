// moe_layer_decode_resident_noalloc(): one MoE block (paper section 2, Eq. 1-3) over experts that all sit in
// device memory, for callers that cannot allocate (code under HIP graph capture, tight serving loops).
//
// It is moe_layer_decode() on a cache that holds every expert, without the cache object: the same kernels run
// (router + gating + lookups + grouping, expert FFN, combine), and everything they need beyond the caller's
// inputs and outputs - the (trivial) cache table, the per-call tables, the arrival counter, the call record and
// the partial sums of the expert kernels - lives in one file-scope device array.  No hipMalloc, hipFree or
// allocating library call is made, here or in the launch helpers.
//
// Every call on a GPU uses that GPU's copy of the array and rewrites the parts that must start from a known
// state, so calls on one GPU must not overlap (different streams without ordering race).
#include <mutex>

#include "moe_internal.hpp"

using namespace moe;

namespace {

constexpr size_t kScratchBytes = MOE_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

// Host code never uses this name as an address: it is resolved per device with hipGetSymbolAddress below.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_mu;
unsigned char* g_ptr[kMaxDevices] = {};     // device address of `scratch` on each GPU
uint32_t g_seq[kMaxDevices] = {};

size_t up(size_t v) { return (v + 255) / 256 * 256; }

// The table of a cache that already holds every expert: expert e in slot e and buffer e, no free buffer.
__global__ void resident_table_kernel(LayerState st, int E, int32_t* arrive, int32_t* n_groups) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < E) {
    st.expert_in[i] = i;
    st.tick[i] = (uint64_t)(i + 1);
    st.buf_of_slot[i] = i;
    st.score[i] = 0.0;
    st.free_buf[i] = -1;
    st.zombie[i] = -1;
    st.used_stamp[i] = 0;
  }
  if (i == 0) {
    st.scalars[SC_CLOCK] = E;
    st.scalars[SC_NRES] = E;
    st.scalars[SC_NFREE] = 0;
    st.scalars[SC_NZOMBIE] = 0;
    st.scalars[SC_CALLSEQ] = 0;
    st.scalars[SC_TRACE_N] = 0;
    *arrive = 0;
    *n_groups = 0;
  }
}

#define HIPCHK(expr)                                                                        \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) return fail(MOE_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

}  // namespace

extern "C" int moe_layer_decode_resident_noalloc(const moe_resident_layer_t* L, const void* x_dev,
                                                 const float* logit_bias_dev, int32_t batch, void* y_dev,
                                                 int32_t* topk_idx_dev, float* topk_w_dev, void* hip_stream) {
  if (!L) return fail(MOE_ERR_INVALID_ARG, "null layer description");
  const int E = L->n_experts, K = L->top_k, d = L->d_model, f = L->d_ff, ns = L->n_shared;
  if (E < 1 || E > 1024) return fail(MOE_ERR_INVALID_ARG, "n_experts must be in 1..1024");
  if (ns < 0 || ns > 64) return fail(MOE_ERR_INVALID_ARG, "n_shared must be in 0..64");
  if (K < 1 || K > E || K > 64) return fail(MOE_ERR_INVALID_ARG, "top_k must be in 1..min(n_experts,64)");
  if (d < 1 || f < 1) return fail(MOE_ERR_INVALID_ARG, "d_model and d_ff must be positive");
  if (L->dtype != MOE_DTYPE_FP32 && L->dtype != MOE_DTYPE_BF16) return fail(MOE_ERR_INVALID_ARG, "unknown dtype");
  if (L->norm_topk != 0 && L->norm_topk != 1) return fail(MOE_ERR_INVALID_ARG, "norm_topk must be 0 or 1");
  if (L->pool_layout != MOE_LAYOUT_ROWMAJOR && L->pool_layout != MOE_LAYOUT_TILED &&
      L->pool_layout != MOE_LAYOUT_TILED_INT4)
    return fail(MOE_ERR_INVALID_ARG, "unknown pool_layout");
  if (!L->router_w || !L->experts) return fail(MOE_ERR_INVALID_ARG, "router_w and experts must not be null");
  if ((ns > 0) != (L->shared_w != nullptr))
    return fail(MOE_ERR_INVALID_ARG, "shared_w must be given exactly when n_shared > 0");
  if (!x_dev || !y_dev) return fail(MOE_ERR_INVALID_ARG, "x_dev and y_dev must not be null");
  if (batch < 1 || batch > (1 << 20)) return fail(MOE_ERR_INVALID_ARG, "batch out of range");
  if (d % (L->dtype == MOE_DTYPE_FP32 ? 4 : 8) != 0)
    return fail(MOE_ERR_UNSUPPORTED, "d_model must be a multiple of %d for this dtype", L->dtype == MOE_DTYPE_FP32 ? 4 : 8);
  if (L->pool_layout == MOE_LAYOUT_TILED && (L->dtype != MOE_DTYPE_BF16 || d % 32 != 0 || f % 32 != 0))
    return fail(MOE_ERR_UNSUPPORTED, "the tiled layout is bf16 only and needs d_model and d_ff to be multiples of 32");
  if (L->pool_layout == MOE_LAYOUT_TILED_INT4 && (L->dtype != MOE_DTYPE_BF16 || !ffn_fused_q4_supported(d, f, 1)))
    return fail(MOE_ERR_UNSUPPORTED, "INT4 experts need bf16 activations, d_model %% 256 == 0 and d_ff %% 32 == 0");
  if ((reinterpret_cast<uintptr_t>(L->router_w) | reinterpret_cast<uintptr_t>(L->experts) |
       reinterpret_cast<uintptr_t>(L->shared_w) | reinterpret_cast<uintptr_t>(x_dev)) & 15)
    return fail(MOE_ERR_INVALID_ARG, "router_w, experts, shared_w and x_dev must be 16-byte aligned");

  const uint64_t eb = moe_expert_block_bytes(d, f, L->dtype, L->pool_layout);
  const int KS = K + ns;
  const size_t NP = (size_t)batch * KS;
  const int G = (int)std::min<size_t>((size_t)batch * K, (size_t)E) + ns;
  const size_t max_miss = std::max<size_t>((size_t)batch * K, (size_t)E);
  FfnPlan plan = plan_ffn(L->pool_layout, d, f, batch);

  // ---- carve the array ----
  size_t o_tick, o_score, o_scal, o_ein, o_bos, o_free, o_zom, o_used, o_idx, o_wp, o_pb, o_sp, o_po, o_gd, o_ng,
      o_arr, o_mail, o_miss, o_h, o_o;
  auto carve = [&]() {
    size_t o = 0;
    o_tick = o; o += up((size_t)E * 8);
    o_score = o; o += up((size_t)E * 8);
    o_scal = o; o += up((size_t)SC_COUNT * 8);
    o_ein = o; o += up((size_t)E * 4);
    o_bos = o; o += up((size_t)E * 4);
    o_free = o; o += up((size_t)E * 4);
    o_zom = o; o += up((size_t)E * 4);
    o_used = o; o += up((size_t)E * 4);
    o_idx = o; o += up((size_t)batch * K * 4);
    o_wp = o; o += up(NP * 4);
    o_pb = o; o += up(NP * 4);
    o_sp = o; o += up(NP * 4);
    o_po = o; o += up(NP * 4);
    o_gd = o; o += up((size_t)G * sizeof(GroupDesc));
    o_ng = o; o += 256;
    o_arr = o; o += 256;
    o_mail = o; o += up(sizeof(Mailbox));
    o_miss = o; o += up(max_miss * sizeof(MissEntry));
    o_h = o; o += plan.fused ? 0 : up(NP * (size_t)f * 4);
    o_o = o;
    o += up(plan.fused ? NP * (size_t)(f / 32) * d * 4 : NP * (size_t)d * 4);
    return o;
  };
  size_t o = carve();
  if (o > kScratchBytes && plan.fused) {
    // the single-launch kernels keep one partial row per 32 rows of d_ff; when those do not fit, the two-pass
    // grouped GEMM (one row per pair) does the same work in a fraction of the scratch
    plan.fused = false;
    plan.gemm = plan.tiled;
    o = carve();
  }
  if (o > kScratchBytes)
    return fail(MOE_ERR_UNSUPPORTED,
                "batch %d of this layer shape needs %zu bytes of scratch; the allocation-free entry point has %zu",
                batch, o, kScratchBytes);
  if (route_cache_lds_bytes(E, E, E, ns, (int)std::min<size_t>(batch, kStageMaxPairs / KS), K, KS) > 64 * 1024)
    return fail(MOE_ERR_UNSUPPORTED, "cache table of this size does not fit in LDS");

  // ---- this GPU's copy of the array ----
  int dev = 0;
  HIPCHK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(MOE_ERR_UNSUPPORTED, "device ordinal %d not supported", dev);
  unsigned char* base = nullptr;
  uint32_t seq = 0;
  {
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_ptr[dev]) {
      void* p = nullptr;
      HIPCHK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
      if (!p) return fail(MOE_ERR_HIP, "hipGetSymbolAddress returned a null address");
      g_ptr[dev] = static_cast<unsigned char*>(p);
    }
    base = g_ptr[dev];
    seq = ++g_seq[dev];
  }

  LayerState st{};
  st.tick = reinterpret_cast<uint64_t*>(base + o_tick);
  st.score = reinterpret_cast<double*>(base + o_score);
  st.scalars = reinterpret_cast<int64_t*>(base + o_scal);
  st.expert_in = reinterpret_cast<int32_t*>(base + o_ein);
  st.buf_of_slot = reinterpret_cast<int32_t*>(base + o_bos);
  st.free_buf = reinterpret_cast<int32_t*>(base + o_free);
  st.zombie = reinterpret_cast<int32_t*>(base + o_zom);
  st.used_stamp = reinterpret_cast<uint32_t*>(base + o_used);
  st.trace = nullptr;
  CallTables t{};
  t.idx = reinterpret_cast<int32_t*>(base + o_idx);
  t.wpair = reinterpret_cast<float*>(base + o_wp);
  t.pair_buf = reinterpret_cast<int32_t*>(base + o_pb);
  t.sorted_pair = reinterpret_cast<int32_t*>(base + o_sp);
  t.pos_of = reinterpret_cast<int32_t*>(base + o_po);
  t.grp = reinterpret_cast<GroupDesc*>(base + o_gd);
  t.n_groups = reinterpret_cast<int32_t*>(base + o_ng);
  int32_t* arrive = reinterpret_cast<int32_t*>(base + o_arr);

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipLaunchKernelGGL(resident_table_kernel, dim3((E + 255) / 256), dim3(256), 0, s, st, E, arrive, t.n_groups);
  HIPCHK(hipGetLastError());

  RouteArgs ra{};
  ra.x = x_dev; ra.router_w = L->router_w; ra.bias = logit_bias_dev;
  ra.d = d; ra.norm_topk = L->norm_topk;
  ra.user_idx = topk_idx_dev; ra.user_w = topk_w_dev;
  ra.arrive = arrive;
  CacheCallArgs a{};
  a.mode = 0; a.B = batch; a.K = K; a.KS = KS; a.E = E; a.C = E; a.P = E; a.n_shared = ns;
  a.policy = MOE_POLICY_LRU; a.gamma = 0.0; a.trace_cap = 0; a.seq = seq;
  a.mailbox = reinterpret_cast<Mailbox*>(base + o_mail);
  a.miss_list = reinterpret_cast<MissEntry*>(base + o_miss);
  a.max_miss = (int32_t)max_miss;
  HIPCHK(launch_route_cache(s, L->dtype, ra, st, t, a, KernelEvents{}));

  FfnArgs fa{};
  fa.x = x_dev;
  fa.buffers = static_cast<const char*>(L->experts);
  fa.shared = static_cast<const char*>(L->shared_w);
  fa.expert_bytes = eb;
  fa.P = E; fa.d = d; fa.f = f; fa.KS = KS;
  fa.g_max = G;
  fa.max_count = batch;
  fa.t = t;
  fa.h = base + o_h;
  fa.o = reinterpret_cast<float*>(base + o_o);
  fa.fused = plan.fused ? 1 : 0;
  fa.pass = 2;
  HIPCHK(launch_ffn(s, L->dtype, plan, fa, KernelEvents{}, KernelEvents{}));
  HIPCHK(plan.fused ? launch_combine_chunks(s, fa.o, t.wpair, t.pos_of, batch, KS, d, f / 32, y_dev)
                    : launch_combine(s, L->dtype, fa.o, t.wpair, t.pos_of, batch, KS, d, y_dev));
  return MOE_OK;
}
