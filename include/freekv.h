/* freekv.h -- C ABI of the MI355X retrieval-decode library.
 *
 * One decode step of one layer, as the paper states it:
 *   - attention of head h over its KV head m = h / G           (Sec. 2.1)
 *   - a budget of B tokens: S sink + W window tokens always kept, the other
 *     (B - S - W) / p pages picked per KV head, the same pages for the whole
 *     query group                                               (Sec. 2.1, 3.2)
 *   - pages are scored through their min-max key summaries, softmax over
 *     pages, mean over the group, top-k                         (Sec. 3.2)
 *   - the step attends with the pages picked at the previous step, unless the
 *     group-mean cosine similarity of this step's and the previous step's
 *     queries is below tau, in which case that KV head re-selects first
 *                                                               (Sec. 3.2, 3.3)
 *   - with the whole KV cache in host memory, picked pages that are not in the
 *     GPU page cache are recalled as one contiguous 2*p*d block per
 *     (page, KV head)                                           (Sec. 4.1, 4.2)
 *
 * Conventions
 *   - Every function returns 0 on success or a negative FKV_E* code; nothing
 *     throws or aborts.  fkv_last_error() gives a text for the last failure.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host
 *     addresses.  `stream` arguments are hipStream_t passed as void*
 *     (NULL = the default stream).  Calls only enqueue work on the stream
 *     unless stated otherwise.
 *   - Element type T of q/K/V is cfg.dtype (2 bytes).  Attention output is fp32.
 *   - One context, one calling thread.  Calls on one context that overlap in
 *     time on different streams are only safe as fkv_decode_step issues them.
 *   - The caller owns q/k/v/out buffers, both arenas and the streams; arenas
 *     must outlive the context.  The library owns what it carves from them.
 */
#ifndef FREEKV_H
#define FREEKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FKV_OK       0
#define FKV_EINVAL  -1   /* bad configuration or argument                         */
#define FKV_ESTATE  -2   /* call order (e.g. attention before any selection)      */
#define FKV_ERANGE  -3   /* layer / page / token count out of range               */
#define FKV_ENOMEM  -4   /* arena too small                                       */
#define FKV_EHIP    -5   /* a HIP call failed; see fkv_last_error                 */
#define FKV_ETIMEOUT -6  /* a kernel gave up a bounded wait for another block     */

#define FKV_DTYPE_FP16 0
#define FKV_DTYPE_BF16 1

#define FKV_PLACE_HBM  0  /* whole KV cache resident in HBM, pages read in place   */
#define FKV_PLACE_HOST 1  /* whole KV cache in a pinned host pool; HBM holds sink,
                             window and a double-buffered cache of picked pages    */

/* how fkv_recall_pages moves a missing page (placement HOST) */
#define FKV_RECALL_GATHER  0  /* a kernel reads the pinned pool through its device address;
                                 page ids never leave the device, no host synchronisation       */
#define FKV_RECALL_MEMCPY  1  /* one hipMemcpyAsync per 16 KiB unit on the copy stream; the miss
                                 list is first copied to the host and the call BLOCKS on it      */

/* Pooling of the page selection over the G query heads of a KV head (App. B.2).  MEAN_S is
 * the method (Sec. 3.2): mean of the per-head softmax over the candidate pages.  MAX_S: their
 * maximum.  MEAN_QK / MAX_QK: mean / maximum of the page weights themselves.  MEAN_Q / MAX_Q:
 * page weights of the channel-wise mean / maximum query of the group. */
#define FKV_POOL_MEAN_S   0
#define FKV_POOL_MAX_S    1
#define FKV_POOL_MEAN_QK  2
#define FKV_POOL_MAX_QK   3
#define FKV_POOL_MEAN_Q   4
#define FKV_POOL_MAX_Q    5
/* Pooling of the query similarity C_i over the group before the test against tau (Sec. 3.3;
 * alternatives of App. B.3): mean (the method), maximum, minimum. */
#define FKV_CORR_MEAN  0
#define FKV_CORR_MAX   1
#define FKV_CORR_MIN   2

/* which page list sparse attention reads */
#define FKV_USE_ACTIVE   0  /* pages committed at the previous step (reuse)        */
#define FKV_USE_PENDING  1  /* pages picked at this step                           */
#define FKV_USE_BY_FLAG  2  /* per KV head: pending if its correction flag is set  */

/* which KV heads fkv_recall_pending serves */
#define FKV_HEADS_ALL        0
#define FKV_HEADS_FLAGGED    1
#define FKV_HEADS_UNFLAGGED  2

typedef struct fkv_ctx fkv_ctx;

typedef struct {
  int32_t n_layers;
  int32_t batch;           /* requests; all share one context length                */
  int32_t n_q_heads;
  int32_t n_kv_heads;      /* G = n_q_heads / n_kv_heads, 1 <= G <= 8               */
  int32_t head_dim;        /* must be 128                                           */
  int32_t page_size;       /* must be 32                                            */
  int32_t max_ctx;         /* multiple of page_size                                 */
  int32_t budget_tokens;   /* B; multiples of page_size, B >= S + W                 */
  int32_t sink_tokens;     /* S                                                     */
  int32_t window_tokens;   /* W                                                     */
  int32_t dtype;           /* FKV_DTYPE_*                                           */
  int32_t placement;       /* FKV_PLACE_*                                           */
  float   tau;             /* correction threshold; <= -1 never corrects, > 1 always */
  int32_t recall_mode;     /* FKV_RECALL_* (placement HOST)                         */
  int32_t select_pooling;  /* FKV_POOL_*: how the selection is pooled over a GQA group */
  int32_t corr_pooling;    /* FKV_CORR_*: how the query similarity is pooled over it   */
} fkv_config;

/* Bytes the library needs: a device arena, and (placement HOST) a pinned,
 * device-mapped host arena for the whole KV pool.  Host pointers in/out. */
int fkv_arena_bytes(const fkv_config* cfg, size_t* dev_bytes, size_t* host_bytes);

/* Create a context on the current device.  dev_arena: device memory, 256-byte
 * aligned, >= dev_bytes.  host_arena: pinned host memory reachable from the
 * device under the same address (hipHostMalloc / torch pin_memory), or NULL
 * for placement HBM.  Zero-fills the device arena (blocking). */
int fkv_create(const fkv_config* cfg, void* dev_arena, size_t dev_bytes,
               void* host_arena, size_t host_bytes, fkv_ctx** out);
int fkv_destroy(fkv_ctx* ctx);
/* Text of the last error of this context (ctx == NULL: of the last failed create). */
const char* fkv_last_error(const fkv_ctx* ctx);
/* Tokens currently cached for `layer` (host-side counter), or a negative code. */
int fkv_context_len(const fkv_ctx* ctx, int32_t layer);

/* Did every kernel of `layer` so far finish its bounded waits?  In the one-launch layer-step the
 * attention blocks of a corrected head wait for that head's selection, made by other blocks of the
 * same launch; the wait is bounded (about 0.1 s).  A block that gives up makes the failure visible
 * on the data path -- every output row of that KV head's query group is NaN -- and sets a flag.
 * With the KV in a host pool the waves that gave up also left page-cache slots unfilled: the outputs of
 * every later step of the layer stay NaN while the flag is up, and after FKV_ETIMEOUT the layer has to
 * be loaded again (fkv_load_prefix) before its results mean anything.
 * That is not expected to happen; this call synchronises the device, returns FKV_ETIMEOUT if it did
 * and clears the flag.  Blocking. */
int fkv_health(fkv_ctx* ctx, int32_t layer);

/* Kernel launches the last fkv_decode_step of `layer` put on the compute stream: 1 when the
 * whole layer-step ran as one launch (selection small enough; with the KV in a host pool also:
 * recall by the gather kernel into the library's own page cache), more otherwise.  The deferred
 * recall on the copy stream is not counted. */
int fkv_step_launches(const fkv_ctx* ctx, int32_t layer);

/* ---- data plane ------------------------------------------------------- */

/* Bulk-load a context of n_tokens (replaces the layer's state): stores K/V in
 * the paged layout, builds the min-max page summaries (Sec. 3.2) and, for
 * placement HOST, writes every page to the host pool in its contiguous
 * per-(page, KV head) unit (Sec. 4.2).  K, V: dev, [batch, n_tokens, n_kv, d]. */
int fkv_load_prefix(fkv_ctx* ctx, int32_t layer, const void* K_dev, const void* V_dev,
                    int32_t n_tokens, void* stream);

/* Append one token per request: k_new, v_new dev [batch, n_kv, d].  Folds the key
 * into the open page's running min/max (Sec. 3.2).  Placement HOST: when the
 * token fills a page, the page is offloaded to the host pool on copy_stream
 * (the transpose happens once, when the page is offloaded -- Sec. 4.2). */
int fkv_kv_append(fkv_ctx* ctx, int32_t layer, const void* k_new_dev, const void* v_new_dev,
                  void* stream, void* copy_stream);

/* Recompute the min-max summaries (channel-wise maximum and minimum of a page's keys, Sec. 3.2
 * "Group-consistent selection") of pages [first_page, first_page + n_pages) from the stored keys;
 * a partial last page is summarised over the tokens it holds.  Placement HBM only (FKV_ESTATE
 * otherwise: the keys are not on the GPU); FKV_ERANGE if the range reaches past the cached context. */
int fkv_page_summary_update(fkv_ctx* ctx, int32_t layer, int32_t first_page, int32_t n_pages,
                            void* stream);

/* ---- the loop's primitives --------------------------------------------- */

/* Correction test (Sec. 3.1, 3.3): per KV head, 1 iff the group-pooled (cfg.corr_pooling;
 * the method: mean) cos(q, q_prev) is < tau, or there is no previous query.  q dev [batch, n_q, d];
 * flags_dev (may be NULL) receives [batch, n_kv] bytes.  Also stages q as the
 * next step's q_prev; it becomes q_prev at fkv_commit. */
int fkv_corr_check(fkv_ctx* ctx, int32_t layer, const void* q_dev, uint8_t* flags_dev, void* stream);

/* Sel(q) for every KV head (Sec. 3.2): scores candidate pages, pools the scores over the query
 * group (cfg.select_pooling; the method: mean of the per-head softmax), picks the
 * k = (B-S-W)/p best (ties to the lower page id).  page_ids_dev (may be NULL)
 * receives [batch, n_kv, k] int32, ascending, padded with -1.  The result is
 * kept as the PENDING selection; for placement HOST the pages it misses in the
 * GPU page cache are worked out too. */
int fkv_page_select(fkv_ctx* ctx, int32_t layer, const void* q_dev, int32_t* page_ids_dev, void* stream);

/* Recall (Sec. 4.1: the data plane moves picked pages from the CPU pool into the GPU cache of selected
 * pages; Sec. 4.2: one contiguous block of 2*p*d elements per (page, KV head)).  Placement HOST; a
 * no-op returning 0 for placement HBM.
 *   page_ids_dev  dev [batch, n_kv, k] int32 or NULL.  A list: ascending, distinct, -1 padded at the end
 *                 (what fkv_page_select emits); it becomes the PENDING selection, as if selected.  Entries
 *                 that are not a full page of the context (negative, or >= context_len / p) are dropped
 *                 (set to -1) on the device, so no address is ever formed from them; an unsorted list only
 *                 costs extra copies.  NULL: the PENDING selection made by fkv_page_select.
 *   head_mask_dev dev [batch, n_kv] bytes or NULL: recall only for heads whose byte is non-zero (NULL = all).
 * Pages of the list that the ACTIVE selection already holds keep their slot and are not copied; the
 * others go to slots that the ACTIVE selection does not reference, so attention on ACTIVE may run
 * beside it.  Everything is enqueued on copy_stream (cfg.recall_mode MEMCPY: blocks on it once);
 * attention on the PENDING selection has to be ordered behind it by the caller (same stream or an
 * event).  FKV_ESTATE with NULL ids before any fkv_page_select. */
int fkv_recall_pages(fkv_ctx* ctx, int32_t layer, const int32_t* page_ids_dev, const uint8_t* head_mask_dev,
                     void* copy_stream);

/* The same for the PENDING selection with the heads chosen by the correction flags (Sec. 3.3:
 * corrected heads are recalled before this step's attention, the others afterwards, for the next
 * step): heads = FKV_HEADS_*.  This is what fkv_decode_step issues. */
int fkv_recall_pending(fkv_ctx* ctx, int32_t layer, int32_t heads, void* copy_stream);

/* o_h = softmax(q_h K^T / sqrt(d)) V over sink + picked pages + window + open
 * page (Sec. 2.1), the group sharing its KV head's pages.  `use` = FKV_USE_*.
 * q dev [batch, n_q, d]; out_dev [batch, n_q, d] fp32. */
int fkv_sparse_decode_attn(fkv_ctx* ctx, int32_t layer, const void* q_dev, float* out_dev,
                           int32_t use, void* stream);

/* fkv_sparse_decode_attn for callers that cannot allocate device memory or hand over a workspace
 * sized for it: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels and the same result, but the split partials, their (max, sum) pairs and
 * the last-block counters live in a static device array of FKV_STATIC_SCRATCH_BYTES that the library
 * itself holds on every GPU it runs on (until the process ends), not in the caller's arena.  The call
 * allocates nothing (no hipMalloc / hipFree, no allocating library routine) and clears what must
 * start at zero with a small kernel, so it may be captured.  A shape whose partials do not fit
 * (heads x splits x G x (d + 2) x 4 bytes, splits as chosen for the shape) is refused with FKV_ENOMEM
 * and a message that names both sizes.  Every call on one GPU shares that GPU's array: calls that
 * overlap in time on one GPU (different streams, different contexts) race; serialise them. */
#define FKV_STATIC_SCRATCH_BYTES (2u << 20)
int fkv_sparse_decode_attn_static(fkv_ctx* ctx, int32_t layer, const void* q_dev, float* out_dev,
                                  int32_t use, void* stream);

/* The hybrid layouts taken literally (Sec. 4.2, "Hybrid layouts" / "Streamed recall"): convert the pages
 * that sparse attention would read with selector `use` (FKV_USE_*) into an NHD-layout pool for a
 * kernel that wants tokens with all KV heads side by side.
 *   nhd_pool_dev   [batch, n_slots, 2 (K, V), page_size, n_kv, d] of the storage type, device,
 *                  16-byte aligned, written completely;
 *   slot_pages_dev [batch, n_kv, n_slots] i32, device: the page held by each slot of each head.
 * Slot s of head m is position s of m's attend list: sink pages, the k selected pages in the order
 * of the page ids (an unused id leaves the slot empty), window pages, the open page.  Empty slots
 * have page -1 and zeros; so have the tokens of the open page beyond the context.
 * n_slots must be budget_tokens / page_size + 1.  Placement HOST: ordered behind the recall of the
 * pages it reads, so it may run on the copy stream right behind fkv_recall_pages.  Asynchronous. */
int fkv_export_nhd(fkv_ctx* ctx, int32_t layer, int32_t use, void* nhd_pool_dev, int32_t* slot_pages_dev,
                   int32_t n_slots, void* stream);

/* Streamed recall into an NHD pool (Sec. 4.2 "Hybrid layouts" / "Streamed recall"): the paper keeps the GPU
 * pool in NHD and converts every recalled per-(page, head) unit on its way in, through two staging buffers,
 * so that the transfer of one unit overlaps the conversion of the one before.  While a pool is attached
 * (placement HOST, recall_mode GATHER; FKV_ESTATE otherwise), every recall of this context does exactly
 * that: a recalled unit goes from the pinned host pool into one of two LDS staging buffers of the recall
 * kernel, from there as 256-byte token rows into the pool (slot = position of the page in its head's attend
 * list) while the next units' transfers are already in flight -- and, unconverted, into its page-cache slot,
 * which is what this library's own attention reads.  fkv_decode_step then also converts the pages of Sel(q_i)
 * that are on the GPU already (sink, window, open page, page-cache hits), so that after the step (and its
 * deferred recall on the copy stream) the pool holds exactly the attend list of the selection the step
 * committed, in the format of fkv_export_nhd.
 *   nhd_pool_dev   dev [batch, n_slots, 2 (K, V), page_size, n_kv, d] of the storage type, 16-byte aligned;
 *   slot_pages_dev dev [batch, n_kv, n_slots] i32;  n_slots must be budget_tokens / page_size + 1.
 * The caller owns both and keeps them alive while attached; nhd_pool_dev == NULL detaches.  One pool serves
 * whichever layer steps (a pool per layer is the caller's to attach before that layer's step).  Host-side
 * switch, nothing is enqueued. */
int fkv_attach_nhd_pool(fkv_ctx* ctx, void* nhd_pool_dev, int32_t* slot_pages_dev, int32_t n_slots);

/* End of step (Sec. 3.3: by the end of a step every KV head's Sel(q_i) has been recalled -- corrected
 * heads before attention, the others deferred -- and is what step i+1 reuses): PENDING becomes ACTIVE,
 * the staged query becomes q_prev.  Host-side flip of two buffer halves, nothing is enqueued.
 * FKV_ESTATE unless fkv_corr_check and fkv_page_select (or fkv_recall_pages with a list) ran since the
 * last commit, and, for placement HOST, unless the pending pages of every head were recalled (a recall
 * with a head mask does not count): the page cache would otherwise hold slots that were never filled. */
int fkv_commit(fkv_ctx* ctx, int32_t layer);

/* One whole step of one layer in the order of Sec. 3.2-3.3:
 * append -> correction test -> selection for all heads -> recall for corrected
 * heads -> attention (corrected heads on the new pages, others on the reused
 * ones) -> deferred recall for the other heads on copy_stream -> commit.
 * No host synchronisation.  copy_stream may equal compute_stream.
 * Small shapes run all of it as one kernel launch (fkv_step_launches); with the KV in a host pool the
 * recall of a corrected head then happens inside its attention -- the wave that attends over a page
 * the cache does not hold reads it from the host pool and puts it into its page-cache slot -- which
 * leaves the same state: by the end of the step the page is cached and was attended over.
 * When the layer-step runs as one launch with the KV in a host pool, the deferred recall is not
 * put on copy_stream at once: the recalls of a quarter of the context's layers (at most 8) are
 * submitted together (one dependency between the two streams instead of one per layer) -- with
 * the last layer of such a group, with the last layer of the context, with the same layer's
 * next step, and by any other call on the context.
 * A caller that wants them on copy_stream now (to synchronise that stream itself) calls fkv_flush. */
int fkv_decode_step(fkv_ctx* ctx, int32_t layer, const void* q_dev, const void* k_new_dev,
                    const void* v_new_dev, float* out_dev, void* compute_stream, void* copy_stream);

/* Submits every deferred recall (Sec. 3.2) that fkv_decode_step has kept back, on the streams of the
 * steps that made them.  Nothing to do is not an error.  Only enqueues. */
int fkv_flush(fkv_ctx* ctx);

/* ---- introspection for tests (blocking: synchronises the device) --------- */
#define FKV_DBG_SUMMARIES   0  /* T     [batch, n_kv, 2 (max,min), max_pages, d]      */
#define FKV_DBG_WEIGHTS     1  /* f32   [batch, n_q, max_pages]  page weights P        */
#define FKV_DBG_SCORES      2  /* f32   [batch, n_kv, max_pages] pooled scores         */
#define FKV_DBG_ACTIVE_IDS  3  /* i32   [batch, n_kv, k]                               */
#define FKV_DBG_PENDING_IDS 4  /* i32   [batch, n_kv, k]                               */
#define FKV_DBG_FLAGS       5  /* u8    [batch, n_kv]                                  */
#define FKV_DBG_MISS        6  /* i32   [batch, n_kv, 1 + k]: count, then page ids     */
#define FKV_DBG_COSINE      7  /* f64   [batch, n_q]                                   */
#define FKV_DBG_TSTAMP      8  /* i64   [64] 100 MHz phase timestamps of head 0, recorded while
                                  fkv_instrument_timestamps (freekv_instrument.h) is on         */
int fkv_debug_read(fkv_ctx* ctx, int32_t layer, int32_t what, void* host_out, size_t bytes);

/* Token-major copy of one page of one (request, KV head): host_out receives
 * K [p, d] then V [p, d] (2*p*d elements of T).  where: 0 = the HBM store
 * (placement HBM), 1 = the host pool, 2 / 3 = the GPU page-cache slot the ACTIVE / PENDING
 * selection holds `page` in (error if it is not picked). */
int fkv_debug_read_page(fkv_ctx* ctx, int32_t layer, int32_t request, int32_t kv_head,
                        int32_t page, int32_t where, void* host_out);

#ifdef __cplusplus
}
#endif
#endif /* FREEKV_H */
