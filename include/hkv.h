/*
 * hkv.h -- C ABI of the HybridKV hot path for AMD MI355X (gfx950).
 *
 * The library implements, as hand-written HIP kernels, the per-head hybrid
 * KV-cache compression of the HybridKV paper (Section 3.3 "Hybrid KV Cache
 * Compression" and Appendix A "Details of Hybrid KV Cache Compression") and the
 * decode attention that runs over the compressed cache:
 *
 *   prefill  (hkv_compress)     static heads: observation-window scoring of the
 *                               prompt (Appendix A, the S_w / s_w equations),
 *                               Top-M historical visual tokens + all historical
 *                               text + the window, compacted into a ragged cache;
 *                               dynamic heads: full K/V adopted into the cache
 *                               and one mean-key summary per fixed-size chunk.
 *   decode   (hkv_decode_attn)  static heads: attention over the compacted rows;
 *                               dynamic heads: query x chunk-summary scores,
 *                               top-k chunks, attention over those chunks' rows;
 *                               tokens generated during decoding are appended
 *                               uncompressed to every head and always attended.
 *
 * Head types (Section 3.1) and per-head budgets (Section 3.2) are INPUTS.
 *
 * Conventions
 *   - Plain C: pointers and sizes only.  Every pointer parameter is marked
 *     [host] or [dev].  [dev] pointers must be 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - The library never allocates or frees device memory: the caller allocates
 *     the cache arena and the workspace with the sizes hkv_query_sizes reports and
 *     owns them.  Q/K/V/out buffers are borrowed for the duration of the call.
 *   - hkv_compress, hkv_decode_attn and hkv_full_decode_attn only enqueue work on
 *     `stream`; they never synchronise and never read device memory on the host.
 *     hkv_cache_create, hkv_cache_export, hkv_cache_import and hkv_cache_rewind
 *     perform small synchronous copies.
 *   - Every function returns an hkv_status (0 = ok, negative = error).  Argument
 *     errors are found on the host before anything is enqueued; on error nothing
 *     is enqueued and no state changes.
 *   - head_dim must be 128; n_q_heads / n_kv_heads (the query group size G) must
 *     be an integer in 1..8.
 *   - Ties in every selection go to the lower index.
 */
#ifndef HKV_H
#define HKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HKV_ABI_VERSION 1u

/* Size of the split-K record array that lives inside the library, one copy per GPU, held from the
 * library's load to the end of the process (see hkv_decode_attn_noalloc). */
#define HKV_NOALLOC_SCRATCH_BYTES (16u << 20)

#ifndef HKV_API
#define HKV_API __attribute__((visibility("default")))
#endif

typedef enum {
  HKV_OK = 0,
  HKV_EINVAL = -1,   /* null pointer, bad struct size / version, bad enum value */
  HKV_ESHAPE = -2,   /* unsupported shape (head_dim, group size, window, chunk size, batch) */
  HKV_EBUDGET = -3,  /* a budget is < 1 */
  HKV_EALIGN = -4,   /* a device pointer is not 16-byte aligned */
  HKV_ENOSPACE = -5, /* caller buffer too small, or the per-head tail is full */
  HKV_ESTATE = -6,   /* call out of order (decode before compress, ...) */
  HKV_EHIP = -7      /* a HIP runtime call failed */
} hkv_status;

typedef enum { HKV_F32 = 0, HKV_BF16 = 1 } hkv_dtype;
typedef enum { HKV_STATIC = 0, HKV_DYNAMIC = 1 } hkv_head_type;

/* What hkv_cache_export / hkv_cache_import move for one (sequence, layer, KV head) unit. */
typedef enum {
  HKV_X_KEPT_IDX = 0,   /* static : int32[retained]  ascending prompt positions kept            */
  HKV_X_SCORES = 1,     /* static : float[C]         s_w of Appendix A                           */
  HKV_X_CHUNK_SEL = 2,  /* dynamic: int32[k]         chunks picked by the last decode step, asc. */
  HKV_X_CHUNK_SIGMA = 3,/* dynamic: float[n_chunks]  chunk scores of the last decode step        */
  HKV_X_CHUNK_MEAN = 4, /* dynamic: dtype[n_chunks][head_dim] chunk summaries                    */
  HKV_X_K_ROWS = 5,     /* dtype[rows][head_dim]: static = compacted rows then tail,
                           dynamic = the whole prompt then tail                                  */
  HKV_X_V_ROWS = 6
} hkv_export_kind;

typedef struct {
  uint32_t struct_size;     /* sizeof(hkv_config) */
  uint32_t abi_version;     /* HKV_ABI_VERSION */
  int32_t n_layers;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;         /* 128 */
  int32_t dtype;            /* hkv_dtype of Q, K, V, out and of the cache */
  int32_t window;           /* w: observation-window length (Appendix A), 1..256, G*w <= 256 */
  int32_t chunk_size;       /* c: tokens per chunk (Appendix A), power of two >= 4; used when
                               hkv_plan.chunk_size is NULL */
  int32_t score_causal;     /* 0: S_w as printed (no mask); 1: window row i sees keys <= C-w+i */
  int32_t max_new_tokens;   /* capacity of every head's uncompressed decode tail */
  float softmax_scale;      /* 0 -> 1/sqrt(head_dim) */
  int32_t decode_tile_rows; /* rows per split-K tile of decode attention: 0 = chosen from the amount of
                               work (a bf16 cache then also carries a second tiling -- 1024-row tiles, or
                               256-row tiles when the first has grown to 1024 -- and every call takes the
                               one that suits its tile count, see hkv_cache_call_tiling); bf16 caches also accept any multiple of 32 from
                               128 to 4096, which every call then uses (tuning knob; the result does
                               not depend on it beyond fp32 summation order) */
  int32_t decode_dynamic;   /* how a decode step is launched: 1 = one workgroup per dynamic head does chunk
                               selection, attention and the output inside the main launch, static heads run as
                               split-K tiles beside them; 2 = chunk selection in the main launch, split-K tiles
                               of the dynamic heads in a second launch; 3 = a single launch of split-K tiles,
                               each dynamic tile repeating its head's chunk selection; 4 (bf16 caches only, else
                               HKV_ESHAPE) = one wide workgroup per head, static or dynamic, does everything
                               for its head and writes the output rows: a single launch without split-K
                               records, for steps whose heads are few (per-layer calls, small batches);
                               5 (bf16 caches with index_generated = 0, else HKV_ESHAPE) = streamed: the rows of
                               all heads of the call form one line of work that is cut into equal shares,
                               one per resident workgroup, each workgroup walking through the heads its share
                               covers (calls over all layers or over one layer; other layer ranges run as 3);
                               0 = chosen when the cache is laid out: 4 for bf16 caches whose heads all have at
                               most 768 rows (tail capacity included); 5 when a call over all layers gives every
                               resident workgroup a share of at least 2048 rows (a call over one layer of such a
                               cache then streams only if its shares reach that length too, else it runs as 3;
                               an explicit 5 streams both); else 3 unless the repeated
                               summary reads would exceed a quarter of a step's bytes, then 2.
                               Under 0, a call that runs as 3 with all its tiles resident at once on a cache
                               with more than 512 chunks per head computes the chunk scores in a small launch
                               of its own ahead of the tiles, which then only pick (same scores, same picks)
                               (tuning knob, same results up to fp32 summation order) */
  int32_t chunk_score_group;/* how the query heads that share a KV head score a chunk (Appendix A gives one
                               query vector per head and does not treat grouped heads): 0 = the inner
                               product of the chunk summary with the SUM of the group's query vectors;
                               1 = the LARGEST of the group's inner products with the chunk summary */
  int32_t index_generated;  /* 0: tokens generated during decoding are kept uncompressed and every head
                               attends all of them (the paper generates at most a few hundred).
                               1 (bf16 caches, decode_dynamic other than 2; else HKV_ESHAPE): a variant for
                               long generations.  On dynamic heads the generated tokens are cut into
                               chunks of the head's chunk size in order of generation; a chunk that was
                               complete before the step has the mean of its keys as its summary and
                               competes with the prompt's chunks for the budget / chunk places (now
                               capped by the chunks there are, generated ones included); the rest of
                               the tail and the step's own token are always attended.  Static heads
                               are not affected.  hkv_cache_export then reports the summaries (and
                               the last step's scores and picks, whose trailing entries may predate
                               that step) of prompt and generated chunks together, prompt first. */
} hkv_config;

/* Per-prompt plan.  All arrays live in HOST memory and are only read during the call. */
typedef struct {
  int32_t batch;               /* number of sequences, 1..4096 */
  const int32_t* cu_seqlens;   /* [host] [batch+1] packed token offsets, cu_seqlens[0] = 0 */
  const uint8_t* is_visual;    /* [host] [total_tokens] 1 = visual token, 0 = text token */
  const uint8_t* head_type;    /* [host] [batch][n_layers][n_kv_heads] hkv_head_type */
  const int32_t* budget;       /* [host] [batch][n_layers][n_kv_heads] tokens, >= 1.
                                  static : total prompt tokens retained, window and historical
                                           text included (Appendix A); values above what exists
                                           are clamped;
                                  dynamic: tokens gathered per step; k = max(1, budget / c)
                                           chunks, at most all chunks */
  const int32_t* chunk_size;   /* [host] [batch] per-sequence chunk size, or NULL */
} hkv_plan;

typedef struct hkv_cache hkv_cache;   /* opaque host-side descriptor */

/* Sizes of the device arena that holds the compressed cache (`cache_bytes`) and of the
 * scratch workspace hkv_compress / hkv_decode_attn need (`workspace_bytes`, the maximum over
 * both calls and any layer range). */
HKV_API int hkv_query_sizes(const hkv_config* cfg, const hkv_plan* plan, size_t* cache_bytes,
                    size_t* workspace_bytes);

/* Lay the cache out inside `cache_dev` ([dev], >= cache_bytes, 256-byte aligned) and upload its
 * descriptor tables (synchronous copy).  *out is a host object freed by hkv_cache_destroy; the
 * device arena stays the caller's. */
HKV_API int hkv_cache_create(const hkv_config* cfg, const hkv_plan* plan, void* cache_dev, size_t cache_bytes,
                     hkv_cache** out);

/* Host-memory tier for the dynamic heads (Section 3.3: a dynamic head keeps its whole prompt K/V
 * outside GPU memory, only the chunk summaries stay resident, and each decode step brings in the
 * chunks it selected).  bf16 caches only (HKV_ESHAPE otherwise).
 *
 * A tiered cache keeps, in the device arena: the static heads' rows, every head's decode tail, the
 * chunk summaries, the selections and the descriptor tables; and in `host_tier`: the prompt rows
 * of the dynamic heads, in the same blocked layout.  hkv_compress writes those rows straight into
 * the host tier, and the decode kernels read the selected chunks' blocks from it in place (the
 * reads travel over the host link while other workgroups of the same launch read device memory),
 * so there is no staging buffer and no copy call.  Results are identical to those of an untiered
 * cache.
 *
 * hkv_query_tier_sizes reports the three sizes for that arrangement.
 * hkv_cache_create_tiered takes, besides hkv_cache_create's arguments,
 *   host_tier [host] >= host_bytes, 256-byte aligned: page-locked host memory that the current
 *             device can address (hipHostMalloc or an allocator built on it).  Pageable memory or a
 *             device pointer -> HKV_EINVAL, found through hipPointerGetAttributes before any kernel
 *             runs.  The call zero-fills it.  The caller owns it and keeps it allocated and
 *             unmodified for the life of the cache.
 * All other entry points take a tiered cache like any other. */
HKV_API int hkv_query_tier_sizes(const hkv_config* cfg, const hkv_plan* plan, size_t* cache_bytes,
                         size_t* host_bytes, size_t* workspace_bytes);
HKV_API int hkv_cache_create_tiered(const hkv_config* cfg, const hkv_plan* plan, void* cache_dev,
                            size_t cache_bytes, void* host_tier, size_t host_bytes, hkv_cache** out);

/* Prefill compression of layers [layer_begin, layer_end) (Section 3.3, Appendix A).
 *   q_window [dev] [n][batch][window][n_q_heads][head_dim]  queries of each sequence's last
 *            `window` prompt positions,
 *   k, v     [dev] [n][total_tokens][n_kv_heads][head_dim]  prompt keys / values,
 * with n = layer_end - layer_begin: the tensors hold exactly the layers of the call, in order.
 * The cache keeps COPIES of what it retains; k and v may be released afterwards. */
HKV_API int hkv_compress(hkv_cache* cache, int layer_begin, int layer_end, const void* q_window, const void* k,
                 const void* v, void* workspace, size_t workspace_bytes, void* stream);

/* One decode step of layers [layer_begin, layer_end).
 *   q            [dev] [n][batch][n_q_heads][head_dim]
 *   k_new, v_new [dev] [n][batch][n_kv_heads][head_dim] or both NULL (no append)
 *   out          [dev] [n][batch][n_q_heads][head_dim]
 * New K/V rows are appended to every head's tail first and take part in this step's attention.
 * Returns HKV_ENOSPACE (nothing enqueued) when a tail would exceed max_new_tokens. */
HKV_API int hkv_decode_attn(hkv_cache* cache, int layer_begin, int layer_end, const void* q, const void* k_new,
                    const void* v_new, void* out, void* workspace, size_t workspace_bytes, void* stream);

/* hkv_decode_attn for callers that can neither allocate device memory nor hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks,
 * kernels and results as hkv_decode_attn, except that the split-K records go to an array of
 * HKV_NOALLOC_SCRATCH_BYTES inside the library (located on the cache's device when the cache was
 * created) instead of a caller workspace.  The call allocates and frees nothing and makes no runtime
 * call besides its kernel launches and a device-id query.
 *   - Returns HKV_ENOSPACE (nothing enqueued) when the records of the call's tiles -- per tile
 *     (n_q_heads / n_kv_heads) * 512 + 64 bytes, tiles as hkv_cache_call_tiling reports them (a streamed
 *     call: one record per workgroup plus one per head of the call) -- exceed the array: use a smaller
 *     layer range or hkv_decode_attn.
 *   - Returns HKV_ESTATE when the current device is not the one the cache was created on.
 *   - All calls on one GPU share that GPU's array: calls that can overlap there (different streams
 *     without an ordering between them, several host threads) race on it and must be serialised by
 *     the caller.  The array keeps the previous call's records; every record a call reads it has
 *     written first, so nothing needs clearing. */
HKV_API int hkv_decode_attn_noalloc(hkv_cache* cache, int layer_begin, int layer_end, const void* q,
                                    const void* k_new, const void* v_new, void* out, void* stream);

/* Uncompressed decode attention over caller-held K/V, the comparison kernel for the decode path:
 * every head attends all tokens of its sequence.
 *   cu_seqlens [host] [batch+1], batch <= 256
 *   q, out     [dev] [n_layers_call][batch][n_q_heads][head_dim]
 *   k, v       [dev] [n_layers_call][total_tokens][n_kv_heads][head_dim]
 * *workspace_bytes of hkv_full_workspace_size tells the scratch it needs. */
HKV_API int hkv_full_workspace_size(const hkv_config* cfg, int32_t batch, const int32_t* cu_seqlens,
                            int n_layers_call, size_t* workspace_bytes);
HKV_API int hkv_full_decode_attn(const hkv_config* cfg, int32_t batch, const int32_t* cu_seqlens,
                         int n_layers_call, const void* q, const void* k, const void* v, void* out,
                         void* workspace, size_t workspace_bytes, void* stream);

/* Forget all appended decode tokens (tail length back to 0); the compressed prompt stays. */
HKV_API int hkv_cache_rewind(hkv_cache* cache, void* stream);

/* Per-unit facts computed on the host at creation (no device access):
 * retained prompt rows (static) or gathered rows k*c (dynamic), number of chunks and k. */
HKV_API int hkv_cache_unit_info(const hkv_cache* cache, int seq, int layer, int head, int32_t* prompt_rows,
                        int32_t* n_chunks, int32_t* k_chunks);

/* Same facts straight from a config and plan, without a cache or a device (host planning only). */
HKV_API int hkv_plan_unit_info(const hkv_config* cfg, const hkv_plan* plan, int seq, int layer, int head,
                               int32_t* prompt_rows, int32_t* n_chunks, int32_t* k_chunks);

/* Bytes of K/V/summary data one decode step of layers [layer_begin, layer_end) must read with
 * `tail` appended tokens per head: sum over static heads of 2*R*(rows + tail) and over dynamic
 * heads of n_chunks*R + 2*R*(k*c + tail), R = head_dim * element size. */
HKV_API int hkv_cache_step_bytes(const hkv_cache* cache, int layer_begin, int layer_end, int tail,
                         uint64_t* bytes);

/* How decode steps of this cache run (decided at creation, see hkv_config.decode_tile_rows and
 * decode_dynamic): *tile_rows = rows per split-K tile, *dynamic_mode = 1 to 5 as described at
 * hkv_config.decode_dynamic.  Either pointer may be NULL. */
HKV_API int hkv_cache_decode_shape(const hkv_cache* cache, int32_t* tile_rows, int32_t* dynamic_mode);

/* The tiling a decode call over layers [layer_begin, layer_end) uses.  bf16 caches under the automatic
 * tile rule (decode_tile_rows = 0) carry a second tiling besides the one that hkv_cache_decode_shape
 * reports.  Where the first has fewer than 1024 rows per tile the second has 1024: a call takes the large
 * tiles when it has more small tiles than the device has compute units and the large tiles give every tile a
 * compute unit of its own (small whole-model steps), the small tiles otherwise (per-layer calls, larger
 * steps).  Where the first has grown to 1024 rows (large caches) the second has 256: a call takes them when
 * its large tiles would not give every compute unit one (calls over few layers).  Same results up to
 * fp32 summation order.  *tile_rows = rows per tile of such a call, *n_tiles = its tiles (tail at
 * full capacity).  A streamed call (dynamic mode 5) reports the rows of a workgroup's share and the number of
 * workgroups instead.  Either pointer may be NULL. */
HKV_API int hkv_cache_call_tiling(const hkv_cache* cache, int layer_begin, int layer_end, int32_t* tile_rows,
                                  int32_t* n_tiles);

/* Tail bookkeeping for callers that record hkv_decode_attn into a HIP graph.  Normally the host mirrors
 * every head's tail length and passes it to the kernels as an argument, which a recorded call would
 * replay unchanged.  With enable = 1 decode calls read and advance the per-layer counters in device
 * memory only, so one recorded call is valid for every replay (three kernels per call instead of two;
 * a full tail is not reported as HKV_ENOSPACE any more: the step then attends without appending).
 * enable = 0 returns to host bookkeeping after reading the counters back (synchronises `stream`).
 * Exports of K/V rows use the host's figure, so switch back before exporting. */
HKV_API int hkv_cache_set_device_tail(hkv_cache* cache, int enable, void* stream);

/* Switches the way decode steps run (1 to 5 as at hkv_config.decode_dynamic); for callers that time them
 * on their own workload and keep the fastest.  Takes effect with the next hkv_decode_attn; the cache
 * content is not touched.  HKV_EINVAL for any other value, HKV_ESHAPE for a value the cache does not
 * support (4 and 5 on an fp32 cache; 2 and 5 on a cache that indexes generated tokens). */
HKV_API int hkv_cache_set_decode_dynamic(hkv_cache* cache, int32_t dynamic_mode);

/* Test / debug access to one unit (synchronises `stream`, then copies).  `dst`/`src` are [host].
 * Export returns HKV_ENOSPACE if `bytes` is smaller than the item; *written gets its size. */
HKV_API int hkv_cache_export(const hkv_cache* cache, int what, int seq, int layer, int head, void* dst,
                     size_t bytes, size_t* written, void* stream);
/* Import overwrites HKV_X_SCORES (static) or HKV_X_CHUNK_SIGMA / HKV_X_CHUNK_MEAN (dynamic). */
HKV_API int hkv_cache_import(hkv_cache* cache, int what, int seq, int layer, int head, const void* src,
                     size_t bytes, void* stream);

/* Stage-isolated runs for selection tests:
 * hkv_compress_from_scores = hkv_compress without the scoring pass (uses the s_w stored in the
 * cache, e.g. after hkv_cache_import); hkv_reselect_chunks re-runs the chunk top-k of the given
 * layers from the stored chunk scores (no append, no attention). */
HKV_API int hkv_compress_from_scores(hkv_cache* cache, int layer_begin, int layer_end, const void* k,
                             const void* v, void* stream);
HKV_API int hkv_reselect_chunks(hkv_cache* cache, int layer_begin, int layer_end, void* stream);

/* Optional per-workgroup time stamps of the main decode launch, for diagnosis (bf16 caches).  With
 * stamps_dev != NULL every later hkv_decode_attn call that runs as the single launch of split-K tiles (launch
 * shape 3, index_generated = 0) runs an instrumented instantiation of that kernel:
 * thread 0 of workgroup b < n_records writes HKV_STAMP_WORDS uint64 words at stamps_dev[HKV_STAMP_WORDS * b]
 * (values of the device's constant 100 MHz counter, 10 ns a tick):
 *   [0] workgroup start, [1] tile descriptor read, [2] chunk selection done (0 for a static tile),
 *   [3] the tile's rows read and its record or output rows written (0: tile not reached at this tail length),
 *   [4] first logical row of the tile, [5] 1 for a dynamic tile, [6] chunk scores in shared memory (dynamic
 *   tiles: between [1] and [2]), [7] 0.
 * Every call overwrites the records; results are unchanged.  Other launch shapes ignore the setting.
 *   stamps_dev : [device, 8-byte aligned] n_records * HKV_STAMP_WORDS uint64, owned by the caller, who keeps it
 *                alive until the setting is cleared with stamps_dev = NULL (then n_records = 0).
 * Errors: HKV_EINVAL (null cache, negative count, buffer without records), HKV_ESHAPE (fp32 cache),
 * HKV_EALIGN. */
#define HKV_STAMP_WORDS 8
HKV_API int hkv_cache_set_stamps(hkv_cache* cache, uint64_t* stamps_dev, int32_t n_records);

/* Optional per-kernel timing of hkv_decode_attn, for benchmarks.  After hkv_profile_enable every
 * decode call on this cache (up to max_calls) attaches a pair of HIP events to each of its kernels
 * (the kernel's own start and stop time stamps; no synchronisation, no extra work on the stream).
 * hkv_profile_read waits for the stream of the profiled calls, returns
 * the summed durations in milliseconds -- ms[0] main launch (chunk scoring and chunk top-k of the
 * dynamic heads together with the split-K attention of the static heads; in dynamic modes 1, 3 and 5
 * also the dynamic heads' attention; in mode 4 the whole step), ms[1] second launch (split-K
 * attention of the dynamic heads in dynamic mode 2; the chunk scores' own launch where the automatic rule
 * puts one ahead of the tiles), ms[2] combination of the split-K tiles (none
 * in mode 4) -- and the number of calls summed,
 * then starts over.
 * hkv_profile_disable releases the events. */
HKV_API int hkv_profile_enable(hkv_cache* cache, int max_calls);
HKV_API int hkv_profile_read(hkv_cache* cache, double* ms, int* n_calls);
HKV_API int hkv_profile_disable(hkv_cache* cache);

/* ---- diagnostic: cumulative focus count of every attention head (paper, Section 2.1, Eq. 1) ---------
 *
 * For one layer and one sequence: at each of n_steps decoding steps every query head attends over the
 * context_len context tokens; F[head][j] counts the steps at which token j was among the head's
 * k = ceil(focus_fraction * context_len) most attended tokens (the paper uses 0.05 and 500 steps).
 * Softmax is increasing, so the ranking is taken on the scaled logits; equal values go to the lower
 * position.  A head whose counts pile up on few tokens is what the paper calls static.
 *   q_steps  : [device] [n_steps][n_q_heads][head_dim]      the layer's queries of the decoding steps
 *   k        : [device] [context_len][n_kv_heads][head_dim] the layer's keys of the context
 *   counts   : [device, 16-byte aligned] [n_q_heads][context_len] int32, overwritten
 *   workspace: [device, 16-byte aligned] at least *min_bytes of hkv_focus_counts_workspace_size (the logits
 *              of one KV head's query heads); with *best_bytes all KV heads go in one pass.
 * Uses cfg's shape, dtype and softmax_scale.  Work is enqueued on `stream`; the call does not
 * synchronise.  (It clears `counts` with a memset on the stream: not meant for graph capture.) */
HKV_API int hkv_focus_counts_workspace_size(const hkv_config* cfg, int32_t n_steps, int32_t context_len,
                                    size_t* min_bytes, size_t* best_bytes);
HKV_API int hkv_focus_counts(const hkv_config* cfg, int32_t n_steps, int32_t context_len, const void* q_steps,
                     const void* k, double focus_fraction, int32_t* counts, void* workspace,
                     size_t workspace_bytes, void* stream);

/* ---- upstream of hkv_compress: head classification and budget allocation ------------------------
 *
 * hkv_head_scores: text-centric sparsity score of every (layer, sequence, KV head) (paper, Section 3.1).
 * Every text token of the prompt (is_visual == 0) attends over the whole prompt with its G query heads,
 * softmax(q K^T * scale) over all keys (with cfg->score_causal = 1 only over keys at or before the
 * token); a row contributes the sum of its k = ceil(focus_fraction * C) largest probabilities (ties at
 * the k-th place counted as often as they fit); the score is the mean over the G*T rows, 0 for a
 * sequence without text.  The paper states k = ceil(0.05 C) for its focus measure; pass 0.05 for that
 * (a double, so that 0.05 * C does not creep over an integer).
 *   cu_seqlens, is_visual : [host] as in hkv_plan
 *   q_prompt : [device] [n_layers_call][total_tokens][n_q_heads][head_dim]  queries of the whole prompt
 *   k        : [device] [n_layers_call][total_tokens][n_kv_heads][head_dim]
 *   scores   : [device] [n_layers_call][batch][n_kv_heads] float
 *   workspace: [device, 16-byte aligned] at least *min_bytes of hkv_head_scores_workspace_size (one head's
 *              intermediate arrays at a time); with *best_bytes all KV heads of a (layer, sequence) go in
 *              one pass.  Contents are scratch.  bf16 inputs with focus_fraction <= 1/18 and sequences of
 *              at most 65536 tokens never write the logits out (the workspace then holds, per text row, the
 *              four largest logits of every 16 keys and a spill list that only rows with long runs of equal
 *              logits touch); other inputs materialise one pass's logits in it.  The sizes cover both.
 * Uses cfg's shape, dtype, softmax_scale and score_causal.  Work is enqueued on `stream`; the call
 * synchronises the stream once at entry (it uploads the text positions).  Not meant for graph capture. */
HKV_API int hkv_head_scores_workspace_size(const hkv_config* cfg, int32_t batch, const int32_t* cu_seqlens,
                                   const uint8_t* is_visual, size_t* min_bytes, size_t* best_bytes);
HKV_API int hkv_head_scores(const hkv_config* cfg, int32_t batch, const int32_t* cu_seqlens, const uint8_t* is_visual,
                    int n_layers_call, const void* q_prompt, const void* k, double focus_fraction, float* scores,
                    void* workspace, size_t workspace_bytes, void* stream);

/* hkv_allocate_budgets: head types and token budgets of one sequence from its sparsity scores (paper,
 * Section 3.1 threshold and Section 3.2, both equations).  Pure host arithmetic on [host] arrays of
 * n_heads entries (all layers and KV heads of the sequence, any order):
 *   head_type[i] = HKV_STATIC if scores[i] >= theta else HKV_DYNAMIC;
 *   B_dyna = ceil(r * (B_total / N) * N_dyna) with r = share_ratio clipped so that B_dyna <= B_total,
 *   B_stat = B_total - B_dyna;
 *   static head: ceil(alpha * B_stat / N_stat + (1 - alpha) * B_stat * score / (sum of static scores));
 *   dynamic head: B_dyna / N_dyna, rounded to the nearest power of two (ties upwards) if pad_pow2 != 0,
 *                 else rounded down.
 * Every ceiling is taken of its argument minus 1e-9, so that a product that is a whole number up to
 * floating-point error does not creep up to the next integer.
 * The budgets feed hkv_plan.budget as they are ("total retained prompt tokens" for static heads).
 * Errors (nothing is written to head_type or budget): HKV_EINVAL for a NaN or negative score or a
 * parameter out of range; HKV_EBUDGET when the total is so small that some head would get less than one
 * token (hkv_plan needs at least one); HKV_ESHAPE when a budget exceeds 2^31 - 1. */
HKV_API int hkv_allocate_budgets(int32_t n_heads, const float* scores, float theta, int64_t total_budget,
                         float share_ratio, float alpha, int32_t pad_pow2, uint8_t* head_type, int32_t* budget);

/* Reference measurement for benchmarks (not part of the method): average duration, in microseconds,
 * of a kernel that only reads `read_bytes` (rounded down to a multiple of 128 KiB) of `buf` [device,
 * 16-byte aligned, buf_bytes long], taken from the kernel's own start/stop time stamps over `reps`
 * launches on `stream` (1..4096; two untimed launches first).  Successive launches walk through
 * `buf`, so give it several times the memory-side cache.  Synchronises `stream` after every launch. */
HKV_API int hkv_probe_stream_read(const void* buf, size_t buf_bytes, size_t read_bytes, int reps, void* stream,
                          double* avg_us);

HKV_API void hkv_cache_destroy(hkv_cache* cache);   /* frees the host descriptor only */
HKV_API const char* hkv_strerror(int status);
HKV_API uint32_t hkv_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HKV_H */
