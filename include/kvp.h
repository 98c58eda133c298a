/*
 * kvp -- block-wise prefill with a fixed-budget KV cache, for AMD MI355X (gfx950).
 *
 * The library follows the statement of the method in Alg. 1 of the paper
 * ("Block-wise Prefill with KV Eviction": input a sequence S, a block size b
 * and a memory budget M; output the compressed KV cache C).  For every block
 * and every layer the caller makes two calls:
 *
 *   kvp_prefill_chunk   the block's queries attend over cache U block
 *                       (Eq. 1, Sec. 2.1) and, when the block will not fit
 *                       into the budget, every candidate key receives its
 *                       importance score (Eq. 4, Sec. 3.2);
 *   kvp_compact         the block is appended to the cache (Alg. 1 line 7)
 *                       and, if the cache now exceeds M, the lowest-scored
 *                       entries are evicted until it holds M (lines 8-11).
 *
 * After the last block kvp_decode_ready hands out the cache (Alg. 1 line 13).
 *
 * General rules
 *  - Every function returns KVP_OK (0) or a negative code.  Nothing throws,
 *    exits, synchronises a stream or allocates device memory: all device
 *    memory is the single buffer the caller passes to kvp_init_cache.
 *  - On KVP_EINVAL, KVP_ESTATE and KVP_ENOMEM no device work has been enqueued
 *    and no state has changed.  KVP_EDEVICE is the exception: the HIP runtime
 *    refused a launch part-way, earlier kernels of the same call may already
 *    be enqueued, and the layer must be treated as lost (free the cache).
 *  - Pointers named q, k, v, out, scores_override and device_buf are DEVICE
 *    pointers; cfg, segs and all out-parameters are HOST pointers.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Work is enqueued on it in call order; the caller orders streams.
 *  - Per layer the calls alternate prefill_chunk, compact, prefill_chunk, ...
 *    and token ranges are consecutive from 0.  A layer is PENDING between
 *    its prefill_chunk and its compact, READY otherwise.
 *  - A kvp_cache is not thread-safe; use one host thread per cache.
 *  - The library reads no environment variable and keeps no global state that
 *    changes results: everything it is told comes through these calls.
 */
#ifndef KVP_H
#define KVP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  KVP_OK = 0,
  KVP_EINVAL = -1,   /* bad argument, shape, layout or null pointer            */
  KVP_ESTATE = -2,   /* call out of order for this layer, or tokens skipped    */
  KVP_ENOMEM = -3,   /* device_buf smaller than kvp_cache_bytes, or host OOM   */
  KVP_EDEVICE = -4   /* the HIP runtime refused a launch or an event call      */
};

enum { KVP_TEXT = 0, KVP_VISUAL = 1 };

/* limits */
enum {
  KVP_MAX_CANDIDATES = 8192,  /* budget + chunk_max may not exceed this        */
  KVP_MAX_SEGMENTS = 64,
  KVP_MAX_TOKENS = 1 << 24    /* longest prefix, in tokens                     */
};

/* One run of consecutive prefix tokens.  Segments must cover [0, N) in order
 * without gaps.  A visual segment is n_planes planes (tiles of an image or
 * frames of a video) of grid_h x grid_w patch tokens, row-major inside a
 * plane, so n_tokens == n_planes * grid_h * grid_w.  Only the merge step reads
 * the grid; with merge off only token_begin / n_tokens matter. */
typedef struct kvp_segment {
  int32_t token_begin;
  int32_t n_tokens;
  int32_t kind;       /* KVP_TEXT or KVP_VISUAL */
  int32_t grid_h;
  int32_t grid_w;
  int32_t n_planes;
  int32_t temporal;   /* 1: adjacent planes are adjacent video frames */
} kvp_segment;

enum {
  KVP_FLAG_DRY_RUN = 1  /* validate and advance the host state machine only:
                           nothing is enqueued, device memory is untouched.
                           For host-side tests of call order and limits. */
};

typedef struct kvp_config {
  int32_t n_layers;
  int32_t n_q_heads;     /* multiple of n_kv_heads                               */
  int32_t n_kv_heads;
  int32_t head_dim;      /* 64 or 128                                            */
  int32_t budget;        /* M of Alg. 1: slots per KV head per layer, >= 1       */
  int32_t chunk_max;     /* b of Alg. 1: most tokens per kvp_prefill_chunk       */
  int32_t merge;         /* 0: eviction only (the paper's method);
                            1: an evicted visual token is first averaged into its
                               best kept grid neighbour (this library's addition) */
  int32_t scratch_sets;  /* how many layers may be PENDING at once (0 means 1);
                            layer l uses set l % scratch_sets                    */
  int32_t flags;         /* KVP_FLAG_*                                           */
  float softmax_scale;   /* 0 means 1/sqrt(head_dim) (Eq. 1)                     */
} kvp_config;

typedef struct kvp_cache kvp_cache;   /* host object, owned by the library */

const char* kvp_strerror(int code);   /* static string, never NULL */

/* Device bytes kvp_init_cache needs for this configuration (persistent cache
 * plus scratch), or 0 if the configuration is invalid.  The persistent part is
 * Eq. 2 at sequence length M plus 8 bytes of metadata per slot. */
size_t kvp_cache_bytes(const kvp_config* cfg);
/* The persistent part alone (K, V, token index, weight). */
size_t kvp_persistent_bytes(const kvp_config* cfg);

/* Create an empty cache (Alg. 1 line 4).  device_buf (256-byte aligned, at
 * least kvp_cache_bytes(cfg) bytes) stays owned by the caller and must outlive
 * the cache; the library carves it up.  Enqueues one small fill kernel on
 * `stream`.  *out receives the host object; release it with kvp_free_cache. */
int kvp_init_cache(const kvp_config* cfg, const kvp_segment* segs, int32_t n_segs,
                   void* device_buf, size_t device_bytes, void* stream, kvp_cache** out);

/* Eq. 1 and Eq. 4 for one block of one layer.
 *   q   [n_tokens, n_q_heads,  head_dim] bf16, contiguous
 *   k,v [n_tokens, n_kv_heads, head_dim] bf16, contiguous
 *   out [n_tokens, n_q_heads,  head_dim] bf16, written
 * Row r attends to every cached entry and to block keys 0..r.  Scores (the
 * softmax weights summed over the block's rows and over the query heads that
 * share a KV head) are left in the layer's scratch set.  k and v must stay
 * valid, in stream order, until kvp_compact for this layer has been enqueued.
 * token_begin must be the layer's next unseen token; 1 <= n_tokens <= chunk_max. */
int kvp_prefill_chunk(kvp_cache* cache, int32_t layer, int32_t token_begin, int32_t n_tokens,
                      const void* q, const void* k, const void* v, void* out, void* stream);

/* The same block, scored the way Sec. 3.2 words it: Eq. 4 is taken with proxy
 * queries from the textual prompt instead of the block's own.
 *   q_obs [n_obs, n_q_heads, head_dim] bf16, contiguous, device; 1 <= n_obs <= chunk_max
 * The attention output is that of kvp_prefill_chunk.  A proxy query sees every
 * candidate (the prompt follows the visual tokens: no causal mask); the scores
 * are the proxy queries' softmax weights summed over them and over the query
 * heads that share a KV head.  Other arguments, state changes and errors as for
 * kvp_prefill_chunk; kvp_compact follows as usual. */
int kvp_prefill_chunk_proxy(kvp_cache* cache, int32_t layer, int32_t token_begin, int32_t n_tokens,
                            const void* q, const void* k, const void* v, void* out,
                            const void* q_obs, int32_t n_obs, void* stream);

/* The same block, scored without any query (the query-agnostic strategy of
 * Sec. 3.2): the anchor is the mean of the candidate keys of a KV head (cache
 * entries and block keys alike), and a key's score is minus its cosine
 * similarity to the anchor, so that the keys that deviate most are kept.
 * The attention output is that of kvp_prefill_chunk; arguments, state changes
 * and errors likewise. */
int kvp_prefill_chunk_keydiff(kvp_cache* cache, int32_t layer, int32_t token_begin, int32_t n_tokens,
                              const void* q, const void* k, const void* v, void* out, void* stream);

/* Alg. 1 lines 7-11 for the block last given to kvp_prefill_chunk(layer).
 * With c cached entries and n block tokens: if c + n <= M all are kept;
 * otherwise each KV head keeps the M candidates with the highest score, equal
 * scores by lower token index.  Kept cache rows stay in their slots; kept block
 * rows, in ascending token order, fill the free slots in ascending order.
 * scores_override: NULL, or device [n_kv_heads, c + n] fp32 (cache slots
 * first, then block tokens) used instead of the computed scores. */
int kvp_compact(kvp_cache* cache, int32_t layer, const float* scores_override, void* stream);

/* kvp_compact (Alg. 1 lines 7-11) for the consecutive layers first_layer ..
 * first_layer + n_layers - 1, every one of them PENDING.  For a model that runs
 * its layers one after the other: kvp_prefill_chunk per layer as the block
 * moves up the stack (the cache needs one scratch set per layer that is pending
 * at a time), then this call once for all of them.  Layers that are in the same
 * state (same entry count, same block, scored the same way -- the case in a
 * prefill) are taken up to 16 at a time by ONE select, ONE merge and ONE move
 * launch, which fills the GPU where a single layer's KV heads cannot; others are
 * taken one by one.  The result is that of n_layers kvp_compact calls, bit for
 * bit.  Every layer's k and v must still be valid.
 *   KVP_EINVAL  bad range;  KVP_ESTATE  a layer of the range is not PENDING
 * (both before anything is enqueued).  KVP_EDEVICE: a launch failed; the layers
 * of the groups launched before it are READY, the rest still PENDING. */
int kvp_compact_layers(kvp_cache* cache, int32_t first_layer, int32_t n_layers, void* stream);

/* One block of the prefix through every layer (the body of the loop of Alg. 1,
 * for all layers): for layer 0 .. n_layers-1, kvp_prefill_chunk (or its proxy or
 * key-only scoring variant) followed by kvp_compact.
 *   q, k, v, out, q_obs   HOST arrays of n_layers DEVICE pointers, shapes as for
 *                         the per-layer calls (q_obs only read for KVP_SCORE_PROXY)
 *   scoring               KVP_SCORE_OWN, KVP_SCORE_PROXY or KVP_SCORE_KEYDIFF
 * The layers go in groups (min(scratch_sets, 16) layers on one stream,
 * scratch_sets / 2 with a side stream): the attention launches of a group one
 * after the other, then, each as ONE launch per kernel for the whole group, the
 * scoring pass of proxy queries or of the keys (the block's own queries are
 * scored inside the attention launch) and the select, merge and move of the
 * compaction.  The results are those of the per-layer calls, bit for bit.
 * With side_stream NULL (or equal to stream) everything is enqueued on `stream`
 * in that order.  With another side_stream every kvp_compact goes there, beside
 * the attention of the layers that follow (in a model nothing after a layer's
 * attention reads the cache being compacted); the library orders the two
 * streams with its own events: a layer's next block waits for that layer's
 * compaction, and a scratch set waits for the compaction of the layer that
 * used it last.  The layers go in groups of scratch_sets / 2 (attention and
 * scoring of a group on `stream`, then its compactions on side_stream), so the
 * streams exchange two events per group; the block's k and v of a layer are read
 * by its compaction on side_stream and must stay valid until then.  That needs
 * scratch_sets >= 2 (KVP_EINVAL otherwise).  Both streams must have the default
 * priority, and between the first such call and kvp_free_cache the per-layer
 * calls must not be mixed in on other streams (the library only orders what it
 * enqueued here).  Errors as for the per-layer calls; layers before the failing
 * one have been enqueued and advanced. */
enum { KVP_SCORE_OWN = 0, KVP_SCORE_PROXY = 1, KVP_SCORE_KEYDIFF = 2 };
int kvp_prefill_block(kvp_cache* cache, int32_t token_begin, int32_t n_tokens,
                      const void* const* q, const void* const* k, const void* const* v, void* const* out,
                      int32_t scoring, const void* const* q_obs, int32_t n_obs,
                      void* stream, void* side_stream);
/* Makes `stream` wait for every compaction kvp_prefill_block has put on
 * side_stream (before the caches are read on `stream`, e.g. for decoding). */
int kvp_prefill_join(kvp_cache* cache, void* stream, void* side_stream);

/* The compressed cache of one layer (Alg. 1 line 13).  Device pointers into
 * device_buf; the first `count` slots of every head are valid; slot order
 * carries no meaning.  KVP_ESTATE while the layer is PENDING. */
typedef struct kvp_view {
  const void* k;              /* [n_kv_heads, budget, head_dim] bf16 */
  const void* v;              /* [n_kv_heads, budget, head_dim] bf16 */
  const int32_t* token_idx;   /* [n_kv_heads, budget]                */
  const float* weight;        /* [n_kv_heads, budget] merge multiplicity, integer-valued */
  int32_t count;
  int32_t budget;
  int32_t next_token;         /* tokens of the prefix seen so far    */
} kvp_view;
int kvp_decode_ready(kvp_cache* cache, int32_t layer, kvp_view* out);

/* One decode step of one layer over the compressed cache (Eq. 1 of Sec. 2.1 with
 * one query row per head; generation reuses the cached keys and values, ibid.).
 * The keys are the layer's `count` cache entries followed by the `n_tail` tokens
 * generated so far, the current token last: the caller keeps that tail, the
 * cache itself is not changed and the layer stays READY.
 *   q       [n_q_heads, head_dim]          bf16, the current token's queries
 *   k_tail  [n_tail, n_kv_heads, head_dim] bf16 (row n_tail - 1 is the current token)
 *   v_tail  same shape
 *   out     [n_q_heads, head_dim]          bf16
 * out[h] = softmax(scale * q[h] . K^T) V over all count + n_tail keys of KV
 * head h / (n_q_heads / n_kv_heads), accumulated in fp32 and rounded once.
 * Uses the layer's scratch set: KVP_ESTATE if the layer is PENDING or another
 * layer's block is pending in that set.  KVP_EINVAL for n_tail < 1, n_tail >
 * 2^20, a null pointer, or more than 16 query heads per KV head. */
int kvp_decode_step(kvp_cache* cache, int32_t layer, const void* q, const void* k_tail, const void* v_tail,
                    int32_t n_tail, void* out, void* stream);

/* kvp_decode_step for callers that cannot allocate and cannot lend scratch memory:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same result (bit for bit when the same number of
 * workgroups per KV head is used, which is the case whenever both calls succeed
 * at the sizes below), but the partial results of the step go to a file-scope
 * device array of KVP_STATIC_SCRATCH_BYTES that the library holds on every GPU
 * it is used on (its address is looked up once per GPU, at kvp_init_cache),
 * not to the layer's scratch set.  The call allocates nothing, synchronises
 * nothing, and does not care whether the scratch set is taken by a pending block
 * (the layer itself must be READY).
 *   KVP_ENOMEM  the step's partial results do not fit: with s = min(128,
 *               ceil((count + n_tail) / 64)) workgroups per KV head wanted, at
 *               least min(s, KVP_STATIC_MIN_SPLITS) sets of n_q_heads *
 *               (head_dim + 2) floats must fit into the array.
 *   KVP_EDEVICE the array's address could not be looked up on this GPU.
 * All calls on one GPU share that GPU's array and every call overwrites what the
 * last one left (nothing in it needs clearing): calls that may overlap on one
 * GPU, on different streams or from different caches, race and must be ordered
 * by the caller.  Other errors as for kvp_decode_step. */
enum { KVP_STATIC_SCRATCH_BYTES = 1 << 20, KVP_STATIC_MIN_SPLITS = 16 };
int kvp_decode_step_static(kvp_cache* cache, int32_t layer, const void* q, const void* k_tail,
                           const void* v_tail, int32_t n_tail, void* out, void* stream);

/* Resume: declare that the caller has written `count` valid slots per head
 * into the layer's K, V, token_idx and weight (through the kvp_view pointers)
 * and that the next block starts at `next_token`.  Layer becomes READY. */
int kvp_set_state(kvp_cache* cache, int32_t layer, int32_t count, int32_t next_token);

/* Tuning and test aid: force one of the attention kernel's three workgroup shapes
 * for every later kvp_prefill_chunk of this cache (0: four waves of 64 rows,
 * 1: four waves of 32 rows, 2: eight waves of 32 rows), or -1 to let the library
 * choose from the launch size again (the default).  Results are the same to
 * rounding; only speed differs.  KVP_EINVAL for any other value. */
int kvp_set_attention_shape(kvp_cache* cache, int32_t shape);

/* Tuning and test aid: where kvp_prefill_chunk takes the scores of Eq. 4 from.
 * 1 (the default): the attention launch itself sweeps its keys a second time once
 * its rows have their normalisers; 0: a separate column-sum kernel after it.  The
 * scores agree to rounding (different summation orders).  Configurations with more
 * than 64 workgroups per KV head always use the separate kernel. */
int kvp_set_score_sweep(kvp_cache* cache, int32_t fused);

/* Scoring passes of kvp_prefill_chunk_proxy and kvp_prefill_chunk_keydiff put off
 * until the compaction.  0 (the default): each call launches its scoring pass
 * itself.  1: the call launches the attention only and leaves the layer PENDING
 * with its scores still to come; kvp_compact or kvp_compact_layers launches them
 * first -- kvp_compact_layers for up to 16 layers of the range per launch, which
 * is what makes it worth while: these passes are launch-sized for one layer.
 * The result is the same bit for bit.  While a layer waits, its q_obs (and, as
 * always, its k and v) must stay valid, and kvp_debug_last has nothing to show
 * for it.  kvp_prefill_block does the same by itself and ignores this setting. */
int kvp_set_deferred_scoring(kvp_cache* cache, int32_t on);

/* Inspection of the last block of a layer (device pointers, valid until the
 * layer's scratch set is reused).  n_cand = c + n of that block; candidates are
 * cache slots 0..c-1 then block tokens.
 *   scores [n_kv_heads, *stride]  fp32, valid after a kvp_compact that had to evict
 *                                 (c + n > budget): the scores it used.  A block that
 *                                 fits into the cache is appended without being scored.
 *   keep   [n_kv_heads, *stride]  uint8, valid after kvp_compact
 *   dst    [n_kv_heads, *stride]  int32 candidate position merged into, or -1
 * Any out-pointer may be NULL. */
int kvp_debug_last(kvp_cache* cache, int32_t layer, const float** scores, const uint8_t** keep,
                   const int32_t** dst, int32_t* n_cand, int32_t* stride);

/* Running totals of what the compactions of this cache have done since
 * kvp_init_cache, kept on the device (a measurement aid: the benchmark turns
 * them into the bytes the compaction kernels had to move).  *totals receives a
 * DEVICE pointer to KVP_T_COUNT unsigned 64-bit counters (NULL for a dry-run
 * cache); read them after synchronising with the streams in use. */
enum {
  KVP_T_EVICTING_HEADS = 0,       /* (layer, KV head) compactions that had to evict          */
  KVP_T_MOVED_ROWS = 1,           /* kept block tokens copied into freed slots (K and V each) */
  KVP_T_MERGE_DESTINATIONS = 2,   /* rows rewritten as a weighted mean                        */
  KVP_T_MERGE_SOURCES = 3,        /* evicted rows averaged into a destination                 */
  KVP_T_COUNT = 4
};
int kvp_debug_totals(kvp_cache* cache, const uint64_t** totals);

/* Per-kernel timing with HIP events on the launching stream.  While enabled
 * every launch is bracketed by two events.  kvp_profile_read waits for the
 * recorded events, adds them up per kernel kind and clears them. */
enum {
  KVP_K_ATTENTION = 0, KVP_K_COLSUM = 1, KVP_K_SELECT = 2, KVP_K_MERGE = 3,
  KVP_K_MOVE = 4, KVP_K_ROWSTAT = 5, KVP_K_KEYDIFF = 6, KVP_K_DECODE = 7, KVP_K_COUNT = 8
};
typedef struct kvp_kernel_stat {
  int64_t launches;
  int64_t layers;     /* layers those launches covered: kvp_prefill_block compacts a group of
                         layers with one launch of each kernel */
  double total_ms;
} kvp_kernel_stat;
int kvp_profile_enable(kvp_cache* cache, int32_t on);
int kvp_profile_read(kvp_cache* cache, kvp_kernel_stat* stats /* [KVP_K_COUNT] */);
const char* kvp_kernel_name(int32_t kind);

/* Measurement aids: what this GPU attains, next to the published peaks.
 * kvp_probe_mfma enqueues `workgroups` workgroups of eight waves that each issue
 * 16 * iters dense 32x32x16 bf16 matrix instructions on register operands (no
 * memory traffic) and leave a checksum per thread in device_out (workgroups *
 * 512 floats); *flops (host) receives the flops of the launch.  kvp_probe_copy
 * enqueues a plain device copy of `bytes` (a multiple of 16, both pointers
 * 16-byte aligned) on `workgroups` workgroups of 256 threads.  The caller times
 * them with events on `stream`.  Neither needs a cache. */
int kvp_probe_mfma(void* device_out, size_t out_bytes, int32_t workgroups, int32_t iters, void* stream,
                   double* flops);
int kvp_probe_copy(void* device_dst, const void* device_src, size_t bytes, int32_t workgroups, void* stream);

void kvp_free_cache(kvp_cache* cache);   /* host object only; NULL is fine */

#ifdef __cplusplus
}
#endif
#endif /* KVP_H */
