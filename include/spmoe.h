/* spmoe.h — C ABI of the MI355X-native SP-MoE hot path.
 *
 * One library, one GPU, one caller thread per context (the library runs one worker thread of its own per
 * context once spmoe_predict_prefetch_async is used).  It implements
 *   (1) the MoE block of the target model on a speculative-verification batch of T tokens
 *       (the N draft tokens plus the last accepted one): gate -> softmax/top-k -> token-to-expert
 *       grouping -> grouped SwiGLU expert FFN -> weighted combination (paper, Eq. 1), and
 *   (2) the speculative expert prefetch that feeds it: experts predicted from draft-stage hidden
 *       states with the target layer's gate (paper, Alg. 1) are copied from pinned host memory into
 *       a per-layer LRU cache of HBM slots on a dedicated copy stream (paper, Alg. 2 and the
 *       "Cache Implementation" paragraph), up to a cutoff layer L.  Experts a verification pass finds
 *       missing are copied on two further streams of the same priority, used alternately, so they share
 *       the link with prefetches still in flight instead of waiting behind them.
 *
 * Conventions
 *   - Every function returns an spmoe_status (SPMOE_OK == 0) and never aborts or throws; on error
 *     the output arguments are left untouched and spmoe_last_error() describes the failure.
 *   - Arguments named dev_*   are device (HBM) pointers owned by the caller.
 *     Arguments named host_*  are ordinary host pointers owned by the caller.
 *     Arguments named pinned_* are page-locked host memory (hipHostMalloc) owned by the caller and
 *     only BORROWED by the library: they must stay allocated until spmoe_destroy().
 *     Hidden states, gates and expert blobs are read with 16-byte vector loads: these pointers must be
 *     16-byte aligned (SPMOE_EINVAL otherwise); rows then stay aligned because d and f are multiples of 32.
 *   - The library owns its cache slots, scratch buffers, its three copy streams and events.
 *   - Kernels run on the compute stream passed to spmoe_create() (a hipStream_t, borrowed; NULL is
 *     the default stream).  Hot-path calls are asynchronous with respect to the device, except
 *     where stated (a few integers of routing are needed on the host when experts are offloaded).
 *   - Cache metadata (which expert sits in which slot, LRU order, statistics) changes in the program
 *     order of the calls (tasks handed to the prefetch worker included); only the copies themselves are
 *     asynchronous.
 *   - Row-major "canonical" tensors: gate Wg[E][d]; expert W_gate[f][d], W_up[f][d], W_down[d][f];
 *     hidden states x[T][d] fp32; outputs out[T][d] fp32.  d and f must be multiples of 32.
 */
#ifndef SPMOE_H
#define SPMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spmoe_ctx spmoe_ctx;

typedef enum {
    SPMOE_OK = 0,
    SPMOE_EINVAL = 1,   /* NULL pointer, bad dtype, bad shape */
    SPMOE_ERANGE = 2,   /* layer / expert / token count / k out of range */
    SPMOE_ENOMEM = 3,   /* host or device allocation failed */
    SPMOE_ESTATE = 4,   /* call not valid in the current state (expert not registered, gate not set ...) */
    SPMOE_EHIP = 5,     /* a HIP runtime call failed */
    SPMOE_ENOTIMPL = 6
} spmoe_status;

typedef enum { SPMOE_F32 = 0, SPMOE_BF16 = 1 } spmoe_dtype;

#define SPMOE_MAX_TOKENS 32    /* upper bound on config.max_tokens */
#define SPMOE_MAX_EXPERTS 128  /* upper bound on n_experts */
#define SPMOE_MAX_SHARED 8     /* upper bound on n_shared */
#define SPMOE_MAX_TOPK 8       /* upper bound on top_k and pred_k */

typedef struct {
    int32_t n_layers;
    int32_t d_model;               /* d */
    int32_t d_ff;                  /* f: expert FFN width */
    int32_t n_experts;             /* E routed experts per layer */
    int32_t top_k;                 /* k of Eq. 1 */
    int32_t n_shared;              /* always-resident shared experts, added with weight 1 */
    int32_t max_tokens;            /* upper bound on T of any call */
    int32_t cache_slots_per_layer; /* HBM budget in experts per layer; == n_experts keeps everything resident */
    int32_t weight_dtype;          /* spmoe_dtype of gate and expert weights */
    int32_t renorm_topk;           /* 1: gating scores of the selected experts renormalised to sum 1 */
    int32_t pred_k;                /* k of Alg. 1's TopK_Index for prediction (1 / 2 / 6 in the paper) */
    int32_t cutoff_layer;          /* L of Alg. 1: predict / prefetch only layers 0..L; < 0 disables */
} spmoe_config;

typedef struct {
    int64_t hits;               /* verify-time: activated expert found cached in HBM (the paper's hit-rate numerator) */
    int64_t misses;             /* verify-time: activated expert not cached -> on-demand load */
    int64_t late_hits;          /* hits whose prefetch copy had not finished when the layer was launched */
    int64_t evictions;
    int64_t prefetch_issued;    /* experts copied by spmoe_prefetch */
    int64_t prefetch_used;      /* ... later used by a verify pass */
    int64_t prefetch_wasted;    /* ... evicted before any use */
    int64_t ondemand_loads;
    int64_t h2d_bytes_prefetch;
    int64_t h2d_bytes_ondemand;
} spmoe_stats;

/* One timed interval recorded while profiling is enabled (times in ms since spmoe_profile_begin). */
typedef struct {
    int32_t kind;      /* 0: verify-layer span (first kernel launch to combine, waits included), 1: prefetch copy,
                          2: on-demand copy, 3: predictor kernel + its result copies, 4: one launch of the two expert
                          GEMMs, 5: routing kernel, 6: combine kernel (3-6: kernels executing), 7 / 8: the compute
                          stream waiting, inside a verify-layer call, for the copy of a cached expert that a
                          prefetch (7) or an earlier on-demand load (8) left in flight, 9: for the on-demand copy of
                          an expert that was missing */
    int32_t layer;
    int32_t expert;    /* copies: expert id; compute spans: number of experts launched */
    int32_t reserved;
    float t_begin_ms;
    float t_end_ms;
} spmoe_profile_record;

/* ---- life cycle -------------------------------------------------------------------------------*/

/* Creates a context: allocates n_layers * cache_slots_per_layer expert slots (plus shared-expert
 * slots) in HBM, scratch for max_tokens tokens, the copy streams and events.  compute_stream is a
 * hipStream_t borrowed for the context's lifetime.  Errors: SPMOE_EINVAL, SPMOE_ERANGE, SPMOE_ENOMEM. */
spmoe_status spmoe_create(const spmoe_config* cfg, void* compute_stream, spmoe_ctx** out);

/* Waits for the compute stream and the copy streams, frees everything the library allocated.  NULL is accepted. */
spmoe_status spmoe_destroy(spmoe_ctx* ctx);

/* Waits until the prefetch worker, the compute stream and the copy streams are idle. */
spmoe_status spmoe_sync(spmoe_ctx* ctx);

/* Human-readable description of the last failure on this context ("" if none; never NULL). */
const char* spmoe_last_error(const spmoe_ctx* ctx);

/* ---- expert storage ---------------------------------------------------------------------------*/

/* Size in bytes of one expert in the library's storage layout: 3*d*f*sizeof(weight) — e.g.
 * 336 MiB for d=4096, f=14336, 16-bit weights, the per-expert size the paper quotes.  0 on bad config. */
size_t spmoe_expert_blob_bytes(const spmoe_config* cfg);

/* Host-side repacking of one expert from canonical row-major matrices into the library's blob
 * layout (bf16: 16x32 MFMA-operand tiles, gate and up interleaved; fp32: the three matrices back to
 * back).  All four pointers are host memory; host_blob_out holds spmoe_expert_blob_bytes().
 * Done once per expert, outside the hot path. */
spmoe_status spmoe_pack_expert(const spmoe_config* cfg, const void* host_w_gate, const void* host_w_up,
                               const void* host_w_down, void* host_blob_out);

/* Gate weights Wg[E][d] of one layer (device memory, weight_dtype, borrowed). */
spmoe_status spmoe_set_gate(spmoe_ctx* ctx, int layer, const void* dev_wg);

/* ---- expert cache: Q_cache + the host store that always keeps every expert ("Cache
 *      Implementation"; evicted experts are overwritten, never copied back) -----------------------*/

/* Registers the pinned host copy (a packed blob) of routed expert (layer, expert).  Borrowed. */
spmoe_status spmoe_expert_cache_register(spmoe_ctx* ctx, int layer, int expert, const void* pinned_blob);

/* Registers shared expert idx of a layer and loads it into its own HBM slot synchronously; it is
 * never evicted and does not count in hit statistics. */
spmoe_status spmoe_expert_cache_register_shared(spmoe_ctx* ctx, int layer, int idx, const void* pinned_blob);

/* Synchronously loads the listed experts of a layer (LRU order as if touched in the given order). */
spmoe_status spmoe_expert_cache_warm(spmoe_ctx* ctx, int layer, const int32_t* host_experts, int n);

/* *host_slot_out = slot index of the expert, or -1 if it is not resident.  Does not touch LRU order. */
spmoe_status spmoe_expert_cache_lookup(spmoe_ctx* ctx, int layer, int expert, int32_t* host_slot_out);

/* Resident experts of a layer in LRU order, head (least recently used) first.
 * host_lru_order_out has room for cache_slots_per_layer entries. */
spmoe_status spmoe_expert_cache_contents(spmoe_ctx* ctx, int layer, int32_t* host_lru_order_out, int32_t* host_n_out);

/* Waits for outstanding work, empties every layer's cache (shared experts stay) and zeroes the statistics. */
spmoe_status spmoe_expert_cache_reset(spmoe_ctx* ctx);

spmoe_status spmoe_expert_cache_stats(spmoe_ctx* ctx, spmoe_stats* host_out);

/* Changes the cutoff layer L of Alg. 1 (same meaning as config.cutoff_layer). */
spmoe_status spmoe_set_cutoff(spmoe_ctx* ctx, int cutoff_layer);

/* ---- hot path ---------------------------------------------------------------------------------*/

/* Gate network + TopK_Index (Alg. 1) + gating scores G(x) of Eq. 1 for T tokens of one layer:
 *   logits[t][e] = sum_j x[t][j] * Wg[e][j]   (fp32, x not rounded)
 *   idx[t][0..k) = the k experts with the largest logits, descending; equal logits -> lower index first
 *   w[t][r]      = softmax(logits[t])[idx[t][r]], divided by their sum over r if renorm_topk
 * dev_idx [T][k] int32, dev_w [T][k] fp32, dev_logits [T][E] fp32 or NULL.  1 <= k <= min(E, SPMOE_MAX_TOPK).
 * Asynchronous on the compute stream. */
spmoe_status spmoe_gate_topk(spmoe_ctx* ctx, int layer, const float* dev_x, int T, int k,
                             int32_t* dev_idx, float* dev_w, float* dev_logits);

/* Token-to-expert grouping of a routing result (the step between gate and experts):
 *   counts[e] = number of assignments a = t*k + r with idx[a] == e; offsets = exclusive prefix sum
 *   (E+1 entries); perm = the assignments listed expert by expert, ascending a inside an expert.
 * All pointers are device memory (int32).  Asynchronous on the compute stream. */
spmoe_status spmoe_token_permutation(spmoe_ctx* ctx, const int32_t* dev_idx, int T, int k,
                                     int32_t* dev_counts, int32_t* dev_offsets, int32_t* dev_perm);

/* Alg. 1 lines 1-6 for n draft-stage hidden states of one layer: if layer <= L, score them with the
 * target layer's gate, take the top pred_k experts per state, rank them most-voted first (ties: larger
 * summed probability, then lower index), keep the first cache_slots_per_layer of that ranking (one task
 * never names more experts than the layer can hold), and drop those already cached, which are moved to
 * the tail of the LRU queue.  The surviving expert ids land in host_ids_out (capacity n_experts) in
 * ranking order; *host_n_out = their number (0 beyond the cutoff).
 * Blocks the calling thread until the few bytes of routing have reached the host. */
spmoe_status spmoe_predict_experts(spmoe_ctx* ctx, int layer, const float* dev_draft_x, int n,
                                   int32_t* host_ids_out, int32_t* host_n_out);

/* Alg. 1 lines 9-10 + Alg. 2 for one layer's task: the listed experts that are not resident are
 * copied, back to back on the prefetch copy stream, into the slots of as many LRU victims; experts that are
 * resident are only moved to the tail of the LRU queue.  A list longer than cache_slots_per_layer is
 * cut to that length.  No-op beyond the cutoff layer.  Returns without waiting for the copies. */
spmoe_status spmoe_prefetch(spmoe_ctx* ctx, int layer, const int32_t* host_experts, int n);

/* Alg. 1 + Alg. 2 without blocking the caller (the paper's worker-thread "Prefetcher"): the predictor
 * for n draft states of `layer` is queued on the compute stream, an event is recorded behind it and the
 * task is pushed to Q_load; a worker thread owned by the context waits for the event, drops cached
 * experts, chooses LRU victims and issues the copies.  No-op beyond the cutoff layer.  Tasks are
 * executed in the order they were queued; every other entry point that reads or changes the cache first
 * waits for the tasks queued before it, so cache contents and statistics are those of the same calls
 * made synchronously.  Errors met by the worker are returned by the next call on the context.
 * dev_draft_x must stay valid until the predictor has run (stream order). */
spmoe_status spmoe_predict_prefetch_async(spmoe_ctx* ctx, int layer, const float* dev_draft_x, int n);

/* Waits until the worker has executed every task queued so far (their copies may still be in flight). */
spmoe_status spmoe_prefetch_drain(spmoe_ctx* ctx);

/* The MoE block of one layer on T tokens (Eq. 1): out[t] = sum_r w[t][r] * FFN_{idx[t][r]}(x[t])
 * (+ shared experts with weight 1).  Experts already cached are computed first; missing ones are
 * loaded on demand (evicting the LRU head) and computed as their copies land.  When every routed
 * expert of the layer is resident the call is fully asynchronous: the host never learns the routing,
 * so that call neither counts hits nor changes the LRU order (nothing can be evicted then anyway).
 * Otherwise it waits for the routing result (T * top_k expert ids) to reach the host before it returns.  The result
 * does not depend on the cache state. */
spmoe_status spmoe_moe_verify_layer(spmoe_ctx* ctx, int layer, const float* dev_x, int T, float* dev_out);

/* The same layer for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): no context, no allocation of any kind, no host wait.
 * Every routed and shared expert must already be in HBM: host_dev_blobs is a HOST array of
 * n_experts + n_shared DEVICE pointers to packed blobs (routed experts 0..E-1, then the shared ones),
 * dev_gate the layer's gate Wg[E][d] in weight_dtype; dev_x [T][d] and dev_out [T][d] are fp32 device
 * memory, all 16-byte aligned; stream is a hipStream_t (NULL = default stream).  Of cfg only the shape
 * fields, weight_dtype, renorm_topk and max_tokens (T <= max_tokens) are used.  The result is bit-identical
 * to spmoe_moe_verify_layer with everything resident (same kernels, same summation order).
 * The intermediates live in one fixed device array of SPMOE_STATIC_SCRATCH_BYTES per GPU, shared by all
 * calls on that GPU: calls that may overlap on one GPU (different streams or threads) race and must be
 * serialised by the caller.  SPMOE_ERANGE if this call needs more than the array holds, roughly
 *   A*f*sizeof(weight) + splits*A*d*4 + T*d*2 + 64 KiB,  A = T*(top_k + n_shared), splits <= 4 K-splits of the down GEMM
 * (5.7 MB for d=6144, f=16384, top-2, T=32).  SPMOE_EINVAL for a bad configuration, NULL or misaligned
 * pointers; SPMOE_EHIP if a launch fails.  Asynchronous on `stream`. */
#define SPMOE_STATIC_SCRATCH_BYTES (16u << 20)
spmoe_status spmoe_moe_layer_resident_static(const spmoe_config* cfg, void* stream, const void* dev_gate,
                                             const void* const* host_dev_blobs, const float* dev_x, int T,
                                             float* dev_out);

/* ---- cutoff-layer policy ("Cutoff layer design") ----------------------------------------------*/

/* Largest cutoff layer L in [0, n_layers) that satisfies the paper's two constraints with k_i
 * approximated by k (the number of experts predicted per layer):
 *     N_expert = (L + 1) * k,    m_peak + N_expert * m_expert < m_gpu                     (memory)
 *     max{ (L - 1) * t_comp + k * t_io,  N_expert * t_io } <= n_layers_draft * t_comp     (overlap)
 * t_comp: per-layer computation time of the drafting stage, t_io: per-expert loading time (same
 * unit); memory sizes in the same unit as each other.  *host_cutoff_out = -1 when not even layer 0
 * can be prefetched under the constraints.  Pure host arithmetic. */
spmoe_status spmoe_suggest_cutoff(int n_layers, int n_layers_draft, int k, double t_comp, double t_io, double m_peak,
                                  double m_expert, double m_gpu, int* host_cutoff_out);

/* Profiles the per-expert loading time the policy needs: copies the registered host blob of
 * (layer, expert) into a temporary HBM buffer `repeats` times on the prefetch copy stream and returns the mean
 * time in ms.  Synchronous; does not touch the cache. */
spmoe_status spmoe_measure_expert_load_ms(spmoe_ctx* ctx, int layer, int expert, int repeats, float* host_ms_out);

/* ---- introspection ----------------------------------------------------------------------------*/

/* How the library tiles the two expert GEMMs of a bf16 configuration (the grouped SwiGLU FFN of Eq. 1) over a
 * workgroup, for batches of cfg->max_tokens tokens: projection 0 = gate/up (contraction over d_model), 1 = down
 * (contraction over d_ff).  Batches of at most 16 tokens use instances that hold one tile of 16 tokens per
 * expert; larger batches use, where the shape has a plan for them, instances of at most 8 waves that take up to
 * 32 tokens of an expert in one pass over its weights (first tile in registers, second tile re-read from the L2
 * cache k-step by k-step).
 * host_plan_out[0] = K-splits across workgroups, [1] = waves that split the K range of one N sub-tile,
 * [2] = k-steps (of 32 elements) per wave, [3] = N sub-tiles side by side in a workgroup, [4] = flags: bit 0
 * set if [0] * [1] * [2] covers the contraction exactly (clear: the generic instance, zero operands past the
 * end), bit 1 set if this projection takes up to 32 tokens of an expert per pass over its weights (clear: 16
 * per pass, so an expert with more tokens streams its weights twice in this projection; only batches of more
 * than 16 tokens can meet that case), [5] = dynamic LDS bytes of the launch.  Pure host arithmetic; SPMOE_EINVAL for a configuration
 * spmoe_create would refuse or for fp32 weights (which do not use these kernels). */
spmoe_status spmoe_gemm_plan(const spmoe_config* cfg, int projection, int32_t host_plan_out[6]);

/* ---- measurement ------------------------------------------------------------------------------*/

/* Starts recording one record per copy, predictor launch and verify-layer call, in issue order.
 *   mode 0: each record is timed with a pair of HIP events on its stream;
 *   mode 1: as 0, plus every kernel launch and every wait for a copy inside the verify-layer calls (kinds 4-9, and
 *           spmoe_last_layer_kernel_ms), which puts events between the kernels and slows the layer down;
 *   mode 2: no events at all: the records only log kind / layer / expert in issue order (times are 0),
 *           e.g. to label the copies of an external trace.
 * spmoe_profile_collect waits for the device, then writes up to cap records and their total number.
 * Leave profiling off when timing throughput. */
spmoe_status spmoe_profile_begin(spmoe_ctx* ctx, int mode);
spmoe_status spmoe_profile_collect(spmoe_ctx* ctx, spmoe_profile_record* host_out, int cap, int* host_n_out);

/* Durations in ms of the kernels of the most recent spmoe_moe_verify_layer call that ran with
 * profiling on: [0] gate/top-k/grouping, [1] gate+up GEMM, [2] down GEMM, [3] combine (summed over
 * launches of that call).  Waits for the compute stream. */
spmoe_status spmoe_last_layer_kernel_ms(spmoe_ctx* ctx, float host_ms_out[4]);

#ifdef __cplusplus
}
#endif
#endif /* SPMOE_H */
