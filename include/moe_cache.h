/*
 * moe_cache.h - C ABI of the MI355X MoE decode step with an offloaded-expert cache.
 *
 * One call to moe_layer_decode() runs one MoE block (paper section 2, Eq. 1-3)
 * on a batch of tokens under expert offloading (section 2, "Expert Offloading
 * Systems"; section 3.2):
 *
 *   router GEMV -> softmax / Top-K gating -> expert-cache lookup with on-demand
 *   host->device fetch of missed experts -> SwiGLU expert FFN over the resident
 *   experts -> weighted combine.
 *
 * Every step runs in HIP kernels on the device named in the config; the host
 * only issues the asynchronous copies of missed experts.  There is no CPU
 * fallback: without a usable GPU every entry point that needs one fails with
 * MOE_ERR_HIP.
 *
 * Conventions
 *   - All functions return MOE_OK (0) or a negative moe_status_t.  Nothing
 *     throws, aborts or prints.  moe_last_error() returns a thread-local,
 *     human-readable description of the last failure on the calling thread.
 *   - "device" pointers are HIP device memory on the cache's device; "host"
 *     pointers are ordinary host memory; "pinned host" is page-locked host
 *     memory from hipHostMalloc (or torch pin_memory).  Borrowed pointers are
 *     never freed by the library and must outlive the cache.
 *   - Streams are passed as void* holding a hipStream_t (NULL = the null
 *     stream).  Kernels of a call are enqueued on the caller's stream; expert
 *     copies run on a stream the library owns.  A call returns once its work
 *     is enqueued; calls that may have to issue copies or to split (see
 *     moe_layer_decode) first wait on the host for the miss list of that call.
 *     Results are valid after the caller synchronises the stream.
 *   - A cache object is not thread-safe; use one thread per cache.  All calls on
 *     one cache share its tables and scratch: issue them on ONE stream, or order
 *     the streams yourself (events) so that calls never overlap on the device.
 */
#ifndef MOE_CACHE_H
#define MOE_CACHE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MOE_OK = 0,
  MOE_ERR_INVALID_ARG = -1,        /* null pointer, size out of range, bad enum value        */
  MOE_ERR_CAPACITY_LT_TOPK = -2,   /* capacity < top_k: one token's experts would not fit    */
  MOE_ERR_OUT_OF_MEMORY = -3,      /* host or device allocation failed                       */
  MOE_ERR_HIP = -4,                /* a HIP runtime call failed (text in moe_last_error)     */
  MOE_ERR_STAGING_EXHAUSTED = -5,  /* no expert buffer left for a load (prefill_pins); the
                                      cache state is left unchanged                          */
  MOE_ERR_UNSUPPORTED = -6,        /* shape / layout combination without a kernel            */
  MOE_ERR_TIMEOUT = -7             /* the device did not report the miss list in time        */
} moe_status_t;

enum { MOE_DTYPE_FP32 = 0, MOE_DTYPE_BF16 = 1 };
enum { MOE_POLICY_LRU = 0, MOE_POLICY_GAMMA = 1 };
enum { MOE_LAYOUT_ROWMAJOR = 0, MOE_LAYOUT_TILED = 1, MOE_LAYOUT_TILED_INT4 = 2 };
/*
 * MOE_FETCH_COPY_ENGINE  hipMemcpyAsync from the pinned pool on the library's copy stream, ordered by events
 *                        before the FFN pass over the fetched experts; the FFN over resident experts overlaps it.
 * MOE_FETCH_IN_KERNEL    small decode calls (up to 6 tokens bf16 - 8 when d_ff >= 4096 -, 16 tokens INT4) on a tiled layout: the expert kernel itself reads a
 *                        missed expert from the pinned pool over PCIe while it computes, and fills the device
 *                        buffer on the way; no copy engine and no host round trip on the miss path.  Calls the
 *                        single-launch kernel does not cover, and prefill_pins, use the copy engine.
 */
enum { MOE_FETCH_COPY_ENGINE = 0, MOE_FETCH_IN_KERNEL = 1 };

typedef struct moe_cache moe_cache_t; /* opaque; owned by the library */

/*
 * Shape and policy of a layer stack.  Notation follows the paper: E experts
 * per layer, K active per token, hidden width d, intermediate width d_ff,
 * cache capacity C resident experts per layer.
 */
typedef struct {
  int32_t n_layers;        /* L >= 1                                                        */
  int32_t n_experts;       /* E, routed experts per layer, 1..1024                          */
  int32_t n_shared;        /* always-resident experts added with weight 1 (0 = none)        */
  int32_t top_k;           /* K, 1..min(E,64)                                               */
  int32_t d_model;         /* d                                                             */
  int32_t d_ff;            /* intermediate width of one expert                              */
  int32_t capacity;        /* C, K <= C; values above E are clamped to E                    */
  int32_t dtype;           /* MOE_DTYPE_*: storage type of weights, x and y                 */
  int32_t norm_topk;       /* 1: gate weights renormalised over the K selected (sum to 1);
                              0: Eq. 2 as printed (softmax over all E, not renormalised)    */
  int32_t policy;          /* MOE_POLICY_LRU: least recently used (gamma -> 0+ limit of
                              Definition C.1); MOE_POLICY_GAMMA: discounted request counts
                              of Definition C.1 with `gamma` (gamma = 1 is LFU)             */
  int32_t max_batch;       /* largest `batch` a call may pass, >= 1                         */
  int32_t staging_buffers; /* spare expert buffers per layer beyond C, >= 0.  Needed only
                              when one call can evict an expert that an earlier token of
                              the same call hit (batch * K > C); batch 1 needs none         */
  int32_t device_id;       /* HIP device ordinal; -1 = the calling thread's current device  */
  int32_t trace_capacity;  /* lookup records kept per layer (0 = tracing off)               */
  int32_t pool_layout;     /* MOE_LAYOUT_*: layout of every expert block (see below)        */
  int32_t fetch_mode;      /* MOE_FETCH_*: how a missed expert reaches its device buffer    */
  double gamma;            /* decay of MOE_POLICY_GAMMA, in [0,1]; ignored for LRU          */
} moe_cache_config_t;

/*
 * Parameters.  All BORROWED for the life of the cache.
 *
 * An expert block holds the three matrices of Eq. 3 for one expert,
 * moe_expert_block_bytes() bytes (3 * d * d_ff * sizeof(dtype) for the first two layouts):
 *   MOE_LAYOUT_ROWMAJOR    W_g [d_ff][d] | W_u [d_ff][d] | W_d [d][d_ff], row-major.
 *   MOE_LAYOUT_TILED       bf16 only; the same values permuted into the order the
 *                          streaming kernels read them (written by moe_pack_expert).
 *   MOE_LAYOUT_TILED_INT4  4-bit group-quantised experts (section 3.2: experts are held in
 *                          INT4 so that more of them stay resident): every run of 32
 *                          consecutive elements along a matrix's contraction dimension
 *                          (d for W_g, W_u; d_ff for W_d) is stored as 32 codes q in 0..15
 *                          and one bf16 scale s and stands for the weights s * (q - 8);
 *                          4.5 bits per weight.  Written by moe_pack_expert_int4.  x, y and
 *                          the router stay bf16 (dtype = MOE_DTYPE_BF16); needs d % 256 == 0,
 *                          d_ff % 32 == 0.  Statistics count bytes of this block size.
 */
typedef struct {
  const void* router_w;    /* device, [L][E][d] row-major, dtype                            */
  const void* expert_pool; /* pinned host, [L][E] expert blocks in one allocation; or NULL  */
  const void* shared_w;    /* device, [L][n_shared] expert blocks; NULL iff n_shared == 0   */
  const void* const* expert_pool_layers; /* or: host array of L pointers, each to one layer's
                              [E] expert blocks in pinned host memory (for stacks whose pool
                              is too large to pin in one piece); the array itself is read
                              only during moe_cache_create.  Exactly one of expert_pool and
                              expert_pool_layers is non-NULL                                */
} moe_weights_t;

typedef struct {
  uint64_t lookups;   /* (token, selected expert) pairs looked up by moe_layer_decode       */
  uint64_t hits;      /* lookups that found the expert resident                             */
  uint64_t misses;    /* lookups that did not; each one is one host->device expert copy     */
  uint64_t evictions; /* resident experts dropped to make room (decode and prefill_pins)    */
  uint64_t pin_loads; /* expert copies issued by moe_cache_prefill_pins                     */
  uint64_t bytes_h2d; /* (misses + pin_loads) * expert_bytes                                */
  uint64_t stream_loads;   /* experts read from the host pool by moe_layer_prefill, not inserted */
  uint64_t bytes_streamed; /* stream_loads * expert_bytes                                    */
} moe_cache_stats_t;

/* One lookup, in the order the lookups were made. */
typedef struct {
  int32_t token;   /* row of the moe_layer_decode call the lookup belongs to                */
  int32_t expert;  /* expert id                                                             */
  int32_t hit;     /* 1 = resident, 0 = fetched                                             */
  int32_t evicted; /* expert dropped to make room, -1 if none                               */
} moe_trace_rec_t;

/* Device-side timing collected while profiling is on (moe_cache_set_profiling). */
typedef struct {
  uint64_t ffn_launches; /* calls without a miss whose two-kernel expert FFN was timed      */
  double ffn_gate_up_ms; /* summed duration of their gate/up kernel                         */
  double ffn_down_ms;    /* summed duration of their down-projection kernel                 */
  uint64_t ffn_fused_launches; /* calls without a miss that used the single-launch decode FFN */
  double ffn_fused_ms;   /* summed duration of that kernel                                  */
  uint64_t route_launches; /* router + gating + cache-lookup launches timed                 */
  double route_ms;       /* their summed duration                                           */
  uint64_t fetch_launches; /* in-kernel fetch: expert-FFN launches that also fetched experts */
  uint64_t fetch_bytes;  /* bytes those launches brought in over PCIe                        */
  double fetch_ms;       /* their summed duration (fetch and compute overlap inside them)   */
  uint64_t decode_single_launches; /* calls without a miss that ran as ONE launch (router, gating, lookups,
                            expert FFN and combine together)                                  */
  double decode_single_ms; /* summed duration of those launches                              */
  uint64_t copies;       /* expert copies timed                                             */
  uint64_t copy_bytes;   /* bytes moved by them                                             */
  double copy_ms;        /* summed duration of the copy batches on the copy stream          */
  uint64_t decode_tiles_launches; /* how many of decode_single_launches ran the tile kernel (one workgroup per
                            compute unit, chosen for one-token calls on large experts) instead of the chunk kernel */
} moe_timing_t;

/* Bytes of one expert block for the given shape; 0 if the arguments are invalid. */
uint64_t moe_expert_bytes(int32_t d_model, int32_t d_ff, int32_t dtype);

/* Bytes of one expert block in the given layout (MOE_LAYOUT_*); 0 if the arguments are invalid. */
uint64_t moe_expert_block_bytes(int32_t d_model, int32_t d_ff, int32_t dtype, int32_t pool_layout);

/*
 * Host-side helper: permute one bf16 expert from MOE_LAYOUT_ROWMAJOR (src, host)
 * into MOE_LAYOUT_TILED (dst, host; may be pinned).  Pure data movement.
 * Requires d_model % 32 == 0 and d_ff % 32 == 0.  src and dst must not overlap.
 */
int moe_pack_expert(const void* src_rowmajor, void* dst_tiled, int32_t d_model, int32_t d_ff);

/*
 * Host-side helper: write one MOE_LAYOUT_TILED_INT4 block (dst_block, host; may be pinned;
 * moe_expert_block_bytes() bytes) from an already quantised expert.  Pure data movement: the
 * quantiser is the caller's.
 *   codes   host, 3 * d * d_ff bytes, one code 0..15 per byte: W_g [d_ff][d] | W_u [d_ff][d] | W_d [d][d_ff]
 *   scales  host, bf16 bits, 3 * d * d_ff / 32 values: S_g [d_ff][d/32] | S_u [d_ff][d/32] | S_d [d][d_ff/32];
 *           element [r][g] scales columns 32 g .. 32 g + 31 of row r
 * Requires d_model % 128 == 0 and d_ff % 32 == 0; a code above 15 is MOE_ERR_INVALID_ARG.
 */
int moe_pack_expert_int4(const uint8_t* codes, const uint16_t* scales, void* dst_block, int32_t d_model,
                         int32_t d_ff);

/*
 * The expert cache of section 2, "Expert Offloading Systems", and section 3.2: per layer, C of the E experts
 * are resident in device memory, the others stay in pinned host memory and are fetched on demand.
 * Create a cache for a layer stack: allocates L * (C + staging_buffers) expert
 * buffers on the device, the per-layer cache tables, scratch for max_batch
 * tokens and a copy stream.  All caches start empty.
 * Errors: INVALID_ARG, CAPACITY_LT_TOPK, UNSUPPORTED (e.g. tiled layout with
 * fp32, widths not multiples of 32), OUT_OF_MEMORY, HIP.  *out is NULL on error.
 */
int moe_cache_create(const moe_cache_config_t* cfg, const moe_weights_t* weights, moe_cache_t** out);

/* Waits for outstanding work of the cache, then frees everything it owns. */
int moe_cache_destroy(moe_cache_t* cache);

/*
 * Empty the cache of one layer (layer = -1: all layers): no expert resident,
 * recency and counts cleared.  Statistics and the trace are kept unless
 * clear_stats != 0.  Ordered after previously enqueued work on `hip_stream`.
 */
int moe_cache_reset(moe_cache_t* cache, int32_t layer, int32_t clear_stats, void* hip_stream);

/*
 * Preload experts before generation (section 3.2: the prefetch set
 * Top-C of the predictor's scores is loaded into the cache before decoding).
 * Equivalent to n lookups in list order that are counted as pin_loads rather
 * than hits or misses; entries already resident are only refreshed; loaded
 * experts remain evictable.  expert_ids: host, n distinct ids in [0,E), n <= C.
 * The copies run on the library's copy stream; `hip_stream` is made to wait for
 * them before the call returns, so later work on that stream sees the experts.
 * Paper anchor for the capacity-C cache this fills: section 2, "Expert Offloading
 * Systems" (a fixed number of experts per layer resident in device memory).
 */
int moe_cache_prefill_pins(moe_cache_t* cache, int32_t layer, const int32_t* expert_ids,
                           int32_t n, void* hip_stream);

/*
 * One MoE block on `batch` tokens (Eq. 1-3 with the offloading runtime).
 *   x_dev          device, [batch][d], dtype; read only
 *   logit_bias_dev device, [batch][E] fp32 added to the router logits; may be NULL
 *   y_dev          device, [batch][d], dtype; written
 *   topk_idx_dev   device, [batch][K] int32, selected experts in ascending id; may be NULL
 *   topk_w_dev     device, [batch][K] fp32 gate weights aligned with topk_idx; may be NULL
 * Tokens are looked up in row order and, within a token, in ascending expert id.
 * A call whose evictions would need more spare buffers than `staging_buffers` provides
 * is executed as consecutive waves of tokens (the batch is halved until every wave
 * fits; one token always fits); routing, hits, misses, evictions and outputs are the
 * same as for the unsplit call, only slower.
 * Host waits: none for batch 1, or for a cache that holds every expert (C >= E), on bf16 experts in the tiled
 * layout with in-kernel fetch (router, gating, lookups and the expert FFN are then one launch, the combine a
 * second one); every other call waits for the device to report the miss list (copy-engine fetch) or whether
 * it has to be split (batched calls on a constrained cache).
 * Errors: INVALID_ARG (null x/y, batch < 1 or > max_batch, layer out of range), HIP, TIMEOUT.
 */
int moe_layer_decode(moe_cache_t* cache, int32_t layer, const void* x_dev,
                     const float* logit_bias_dev, int32_t batch, void* y_dev,
                     int32_t* topk_idx_dev, float* topk_w_dev, void* hip_stream);

/*
 * Prefetch set for a cache shared by several sequences (section 3.2 forms, per layer, the
 * set Top-C of the predictor's scores for one sequence; for a batch of sequences decoded
 * together the scores are summed over the sequences first).  Host-side helper.
 *   scores   host, [n_seqs][n_experts] fp32, summed per expert in fp64 in row order
 *   ids_out  host, [min(capacity, n_experts)]: the selected experts, lowest total first, so
 *            that passing the list to moe_cache_prefill_pins leaves the best-scored expert
 *            most recently used; equal totals rank the lower id higher
 *   n_out    number of ids written
 */
int moe_pooled_prefetch_set(const float* scores, int32_t n_seqs, int32_t n_experts, int32_t capacity,
                            int32_t* ids_out, int32_t* n_out);

/*
 * Prompt processing in streaming mode.  The paper places the prefetch "before generation begins"
 * (section 3.2) and does not say how the prompt's own MoE layers meet the cache; the reading taken here: the
 * n_tokens prompt tokens go through the layer in one call (Eq. 1-3 as in moe_layer_decode), experts that are
 * resident are read from their buffers, every other selected expert is read straight from the pinned host pool
 * by the kernels and is NOT inserted; recency, counts, the trace and hits/misses are left untouched, so a one-off
 * scan over a long prompt does not flush the cache.  Counted as stream_loads / bytes_streamed.
 * Arguments as for moe_layer_decode; n_tokens <= max_batch.  Needs a tiled layout, bf16 or INT4
 * (MOE_ERR_UNSUPPORTED otherwise) and a device-visible pinned expert_pool.
 */
int moe_layer_prefill(moe_cache_t* cache, int32_t layer, const void* x_dev, const float* logit_bias_dev,
                      int32_t n_tokens, void* y_dev, int32_t* topk_idx_dev, float* topk_w_dev, void* hip_stream);

/*
 * Counters of one layer (layer = -1: summed over layers).  `misses` is the N_miss of the paper's latency model
 * (Eq. 4: decode time = compute time + N_miss x transfer time), and, as appendix C.1 notes, the number of cache
 * misses equals the number of host->device expert transfers: bytes_h2d = (misses + pin_loads) x block bytes.
 * Calls that did not wait for the device counted their hits and misses there: the call waits for the device's
 * enqueued work when such calls were made since the cache was created.
 */
int moe_cache_stats(const moe_cache_t* cache, int32_t layer, moe_cache_stats_t* out);

/*
 * Copy up to `max_records` lookup records of one layer, oldest first, into
 * host_out (host).  *n_out = records copied; *n_total (may be NULL) = records
 * produced since the last clear, which exceeds trace_capacity if it overflowed.
 * Waits for the layer's enqueued work.
 */
int moe_cache_read_trace(moe_cache_t* cache, int32_t layer, moe_trace_rec_t* host_out,
                         int64_t max_records, int64_t* n_out, int64_t* n_total);

/* Expert ids resident in one layer, ascending, into host_out[capacity]; *n_out = count. */
int moe_cache_resident(moe_cache_t* cache, int32_t layer, int32_t* host_out, int32_t* n_out);

/* Turn per-kernel HIP-event timing on (1) or off (0); off by default. */
int moe_cache_set_profiling(moe_cache_t* cache, int32_t enabled);

/* Read and optionally clear the timing sums; waits for the timed work. */
int moe_cache_timing(moe_cache_t* cache, moe_timing_t* out, int32_t clear);

/*
 * Calibration, not part of the decode path: time `iters` launches of a plain
 * streaming read (mode 0; dst_dev may be NULL) or a plain copy (mode 1) of
 * `bytes` bytes (a multiple of 16) between device buffers, after one warm-up
 * launch.  *avg_ms = mean kernel time from HIP events attached to each dispatch.
 * The read kernel uses the access pattern of the expert kernels (wave-wide
 * 16-byte loads, all issued before use), so bytes / *avg_ms is the bandwidth the
 * GPU sustains for that pattern; the copy is the reference dispatch for scaling
 * profiler memory counters.
 */
int moe_probe_stream(void* src_dev, void* dst_dev, uint64_t bytes, int32_t mode, int32_t iters,
                     void* hip_stream, double* avg_ms);

/*
 * Cache-simulation loss, forward value (paper section 3.1.1; appendix C.1, Definition C.1 and
 * Proposition C.2).  Not part of the decode path: it scores routing traces, e.g. the idx output of
 * moe_layer_decode collected over a sequence, by how cache-friendly they are.
 *
 * idx_dev   device, int32 [n_traces][T][K]: the K distinct experts requested at each token (the request
 *           vector r^(t), ||r||_1 = K), one trace per (sequence, layer); may be NULL when it holds no element.
 * c1_dev    device, fp64 [n_traces][n_experts]: first cache state c^(1), L1 norm = capacity (for instance
 *           the indicator of a prefetch set); NULL = uniform capacity/n_experts.
 * out_dev   device, fp64 [n_traces][2]: per trace
 *             [0] sum_t <r^(t), 1 - c^(t)> with the soft cache  Gamma^(1) = 1,
 *                 c^(t+1) = (gamma Gamma^(t) c^(t) + r^(t)) / Gamma^(t+1),  Gamma^(t+1) = gamma Gamma^(t) + K/capacity;
 *             [1] sum_t <r^(t), 1 - Chat^(t)>, Chat^(t) = Top-capacity of the discounted counts
 *                 Ctilde^(t+1) = gamma Ctilde^(t) + r^(t), Ctilde^(1) = c^(1), ties to the lower expert id.
 *           L_cs and L_cs^hard are these sums added over the traces and divided by n_traces * T.
 * flag_dev  device, int32 [n_traces]: 0, or 1 if the trace held an id outside 0..n_experts-1 (its sums then
 *           stop at that token).
 * All arithmetic is fp64 in the order written above.  The kernel is enqueued on hip_stream; the call does not
 * wait for it.  Limits: n_experts <= 1024, K <= 64, 0 <= gamma <= 1; violations return MOE_ERR_INVALID_ARG.
 * The library keeps no reference to any argument.
 */
int moe_cache_sim_loss(const int32_t* idx_dev, int32_t n_traces, int32_t T, int32_t K, int32_t n_experts,
                       int32_t capacity, double gamma, const double* c1_dev, double* out_dev, int32_t* flag_dev,
                       void* hip_stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): moe_layer_decode() for a layer whose experts ALL sit in device memory, without a cache
 * object.  The call allocates nothing: the tables and partial sums its kernels need live in one device array of
 * MOE_NOALLOC_SCRATCH_BYTES that the library holds on every GPU it runs on until the process ends.
 *   layer      host; shape of the layer and device pointers to its parameters (all borrowed for the call):
 *              router_w [E][d], experts [E] expert blocks in `pool_layout` (expert e at byte e *
 *              moe_expert_block_bytes()), shared_w [n_shared] blocks or NULL iff n_shared == 0
 *   other arguments as for moe_layer_decode; the device is the calling thread's current device.
 * topk_idx and topk_w equal those of moe_layer_decode on a cache of capacity E preloaded with experts 0..E-1 in
 * that order; y equals it up to the order in which the fp32 partial sums of an expert are added: bit for bit when
 * both entry points run the same expert kernel, within the last bf16 digit otherwise (one-token calls on shapes that
 * moe_layer_decode hands to its tile kernel; batches that this entry point runs through the grouped GEMM so that its
 * partial sums fit the array).
 * Nothing is counted or traced.  A batch whose tables and partial sums exceed the array is rejected with
 * MOE_ERR_UNSUPPORTED (the message names the bytes needed).  All calls on one GPU share the array: calls that
 * overlap in time on one GPU (different streams without ordering, different threads) race.
 */
#define MOE_NOALLOC_SCRATCH_BYTES (32u << 20)
typedef struct {
  int32_t n_experts, n_shared, top_k, d_model, d_ff;
  int32_t dtype;        /* MOE_DTYPE_*                                                          */
  int32_t norm_topk;    /* as in moe_cache_config_t                                             */
  int32_t pool_layout;  /* MOE_LAYOUT_*                                                         */
  const void* router_w; /* device                                                               */
  const void* experts;  /* device                                                               */
  const void* shared_w; /* device or NULL                                                       */
} moe_resident_layer_t;
int moe_layer_decode_resident_noalloc(const moe_resident_layer_t* layer, const void* x_dev,
                                      const float* logit_bias_dev, int32_t batch, void* y_dev,
                                      int32_t* topk_idx_dev, float* topk_w_dev, void* hip_stream);

/* Text of the last error on this thread ("" if none). */
const char* moe_last_error(void);

/* Library version string. */
const char* moe_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MOE_CACHE_H */
