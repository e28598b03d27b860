// Internal declarations shared by the host runtime and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "moe_cache.h"

namespace moe {

// Scalars of one layer's cache table (device, int64 each).
enum { SC_CLOCK = 0, SC_NRES = 1, SC_NFREE = 2, SC_NZOMBIE = 3, SC_CALLSEQ = 4, SC_TRACE_N = 5, SC_COUNT = 8 };

// Device-resident cache table of one layer.  A *slot* is a logical cache entry
// (C of them); a *buffer* is a physical expert-sized block of HBM (P = C +
// staging of them).  A slot owns exactly one buffer while it holds an expert.
struct LayerState {
  int32_t* expert_in;     // [C] expert held by the slot, -1 = empty (slots fill in index order)
  uint64_t* tick;         // [C] value of the layer clock at the slot's last use
  int32_t* buf_of_slot;   // [C]
  int32_t* free_buf;      // [P] stack of unused buffers
  int32_t* zombie;        // [P] buffers released by the previous call, reusable from the next call on
  uint32_t* used_stamp;   // [P] call sequence number of the buffer's last use
  double* score;          // [E] discounted request count (gamma policy)
  int64_t* scalars;       // [SC_COUNT]
  moe_trace_rec_t* trace; // [trace_cap]
};

struct MissEntry { int32_t expert; int32_t buffer; };

// Host-visible record the cache kernel fills for every call (pinned host memory).
struct Mailbox {
  uint32_t seq;        // written last: sequence number of the call this record belongs to
  int32_t status;      // MOE_OK or MOE_ERR_STAGING_EXHAUSTED
  int32_t n_miss;      // expert copies the host has to issue
  int32_t n_evict;
  int32_t n_groups;    // distinct expert buffers used by the call (incl. shared experts)
  int32_t n_hits;
  int32_t pad[2];
};

// One group = the (token, expert) pairs of a call that read the same expert buffer.  A single 32-byte record so
// that an FFN workgroup learns everything it needs to start streaming weights in one memory round trip.
struct __attribute__((aligned(32))) GroupDesc {
  int32_t buf;     // buffer id (>= P: shared expert P + s)
  int32_t begin;   // first position of the group in sorted_pair
  int32_t count;   // pairs in the group
  int32_t miss;    // 1 if the buffer is being filled by this call
  int32_t pair0;   // sorted_pair[begin], the group's first pair (its token is pair0 / KS)
  int32_t expert;  // miss == 1: the expert being brought into the buffer; else -1
  int32_t pad[2];
};

// Per-call scratch tables (device).
struct CallTables {
  int32_t* idx;          // [B][K]  selected experts, ascending id
  float* wpair;          // [B][KS] gate weight per (token, expert) pair; 1 for shared experts
  int32_t* pair_buf;     // [B*KS]  buffer id the pair reads (>= P: shared expert P + s)
  int32_t* sorted_pair;  // [B*KS]  pairs ordered by buffer id, stable
  int32_t* pos_of;       // [B*KS]  inverse of sorted_pair
  GroupDesc* grp;        // [G]     one record per distinct expert buffer of the call
  int32_t* n_groups;     // [1]     number of groups of the call (0 if the call failed)
};

struct CacheCallArgs {
  int32_t mode;          // 0 decode, 1 pin, 2 prompt streaming (cache read-only)
  int32_t B, K, KS, E, C, P, n_shared;
  int32_t policy;
  double gamma;
  int32_t trace_cap;
  uint32_t seq;
  const int32_t* pin_ids; // mode 1: host-mapped list of K ids (B = 1)
  Mailbox* mailbox;       // host-mapped
  MissEntry* miss_list;   // host-mapped, [max_miss]
  int32_t max_miss;
  int32_t row0;           // row of the caller's batch at which this wave of tokens starts (trace records)
};

struct FfnArgs {
  const void* x;           // [B][d]
  const char* buffers;     // layer's expert buffers, P blocks
  const char* shared;      // layer's shared expert blocks (may be null)
  uint64_t expert_bytes;
  int32_t P, d, f, KS;
  int32_t g_max;           // grid rows launched; rows >= *t.n_groups exit at once
  int32_t max_count;       // upper bound on tokens per group (= batch)
  CallTables t;
  void* h;                 // [B*KS][f]  fp32 (row-major path) or bf16 (tiled path)
  float* o;                // [B*KS][d]; fused path: partial sums [pairs][f/32][d]
  int32_t fused;           // 1: o holds per-chunk partial sums (fused decode kernel)
  int32_t pass;            // 0: groups whose buffer was resident, 1: groups fetched by this call, 2: all
  const char* pool;        // in-kernel fetch: this layer's expert blocks in pinned host memory (device-visible)
  int32_t fetch;           // 1: groups with miss == 1 read their weights from `pool` and fill their buffer
  int32_t n_parts;         // tile kernel: workgroups (= partial rows in o) per group
  int32_t work_down;       // grouped GEMM with a work list: offset of the down pass's items in the list (0: no list)
};

// Router inputs of one call.
struct RouteArgs {
  const void* x;          // [B][d]
  const void* router_w;   // [E][d] of this layer
  const float* bias;      // [B][E] or null
  int32_t d, norm_topk;
  int32_t* user_idx;      // optional copies of the routing result for the caller
  float* user_w;
  int32_t* arrive;        // [1] workgroup arrival counter, zero between launches
};

// Everything the single-launch decode kernel needs beyond FfnArgs: it routes and looks up itself.  Every
// workgroup repeats the routing and the lookups from the table `st_in` (read-only during the launch) and reaches
// the same result; one extra workgroup alone writes the table after the call to `st_out` (the layer's other
// copy), the gate weights, the trace, the counters and the call record.  The host swaps the two copies after the
// launch.
struct RoutedArgs {
  RouteArgs r;               // x, router_w, bias, d, norm_topk, user_idx, user_w (arrive unused)
  const void* router_packed; // this layer's router matrix in matrix-core operand order (launch_pack_router)
  LayerState st_in, st_out;
  CacheCallArgs a;
  unsigned long long* dev_stats;  // [3] hits, misses, evictions of the layer, accumulated on the device
  Mailbox* log;              // optional second copy of the call record (host-mapped), for the profiler
};

// Pairs (token, expert) of a call are staged in LDS up to this many; larger calls use global scratch.
constexpr size_t kStageMaxPairs = 2048;

// Optional HIP events bracketing single kernels (attached to the dispatch packets themselves).
struct KernelEvents {
  hipEvent_t start = nullptr, stop = nullptr;
};

size_t route_cache_lds_bytes(int E, int C, int P, int n_shared, int B, int K, int KS);

hipError_t launch_route_cache(hipStream_t s, int dtype, const RouteArgs& r, const LayerState& st, const CallTables& t,
                              const CacheCallArgs& a, KernelEvents ev);
hipError_t launch_pin(hipStream_t s, const LayerState& st, const CallTables& t, const CacheCallArgs& a);
// dev_stats: the layer's device-side counters (hits, misses, evictions), zeroed when non-null
hipError_t launch_reset(hipStream_t s, const LayerState& st, int E, int C, int P, int clear_trace,
                        unsigned long long* dev_stats);
hipError_t launch_ffn_rowmajor(hipStream_t s, int dtype, const FfnArgs& a, KernelEvents gate_up, KernelEvents down);
hipError_t launch_ffn_tiled(hipStream_t s, const FfnArgs& a, KernelEvents gate_up, KernelEvents down);
hipError_t launch_ffn_gemm(hipStream_t s, const FfnArgs& a, KernelEvents gate_up, KernelEvents down);
// Most tokens per call for which the single-launch bf16 decode kernel is used (it can take 16 per expert; the
// whole call is faster with the grouped GEMM from about 6 tokens on: 109 against 110 us at 6, 119 against 133 us
// at 8 on the OLMoE-like layer).
constexpr int kFusedMaxTokens = 6;
// Shapes with a long contraction in the down pass (d_ff >= 4096) keep the single-launch kernel up to 8 tokens: the
// grouped GEMM's down pass is the weaker one there (Phi-like layer: 286 against 337 us at 7 tokens, 312 against 332 us
// at 8; Mixtral-like: 488 against 510 us at 7, level at 8; from 12 tokens on the GEMM wins on both).
inline int fused_max_tokens(int d_ff) { return d_ff >= 4096 ? 8 : kFusedMaxTokens; }
bool ffn_fused_supported(int d, int f, int max_count);
hipError_t launch_ffn_fused(hipStream_t s, const FfnArgs& a, KernelEvents ev);
// Single-launch decode (router + gating + lookups + expert FFN; combine_chunks follows): shapes it covers, and
// the launch.
size_t router_packed_bytes(int E, int d);      // per layer
hipError_t launch_pack_router(hipStream_t s, const void* router_w, void* out, int E, int d, int n_layers);
bool decode_single_supported(int pool_layout, int policy, int E, int C, int P, int n_shared, int K, int d, int f,
                             int batch);
hipError_t launch_decode_single(hipStream_t s, int pool_layout, const FfnArgs& a, const RoutedArgs& ra, KernelEvents ev);
hipError_t launch_decode_single_q4(hipStream_t s, const FfnArgs& a, const RoutedArgs& ra, KernelEvents ev);
// Tile variant of the single-launch decode (one workgroup per compute unit, bf16 experts, one token): workgroups per
// group it would use on a GPU of n_cu compute units, 0 when the chunk kernel is the one to launch.
int decode_tiles_parts(int pool_layout, int d, int f, int batch, int groups, int n_cu, int E);
hipError_t launch_decode_tiles(hipStream_t s, const FfnArgs& a, const RoutedArgs& ra, KernelEvents ev);
int fused_q4_waves(int d);
bool ffn_fused_q4_supported(int d, int f, int max_count);
hipError_t launch_ffn_fused_q4(hipStream_t s, const FfnArgs& a, KernelEvents ev);
hipError_t launch_ffn_gemm_q4(hipStream_t s, const FfnArgs& a, KernelEvents gate_up, KernelEvents down);
// Which expert-FFN kernels run a call of `batch` tokens on experts of the given layout and shape.
struct FfnPlan { bool fused, gemm, tiled, q4; };
FfnPlan plan_ffn(int pool_layout, int d, int f, int batch);
hipError_t launch_ffn(hipStream_t s, int dtype, const FfnPlan& p, const FfnArgs& a, KernelEvents ke1, KernelEvents ke2);
// identity: pair (b, j) has partial row b * KS + j (pos_of is not read)
hipError_t launch_combine_chunks(hipStream_t s, const float* o_part, const float* wpair, const int32_t* pos_of,
                                 int B, int KS, int d, int n_chunks, void* y, bool identity = false);
hipError_t launch_combine(hipStream_t s, int dtype, const float* o, const float* wpair, const int32_t* pos_of,
                          int B, int KS, int d, void* y);

// Launch with the events (if any) attached to the kernel's own dispatch, so that
// hipEventElapsedTime(start, stop) is the kernel's execution time.
template <typename... Args>
inline void launch_timed(void (*kernel)(Args...), dim3 grid, dim3 block, size_t lds, hipStream_t s, KernelEvents ev,
                         Args... args) {
  if (ev.start && ev.stop)
    hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, s, ev.start, ev.stop, 0, args...);
  else
    hipLaunchKernelGGL(kernel, grid, block, lds, s, args...);
}

// Records the text returned by moe_last_error() on this thread and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

}  // namespace moe
