/* oxy.h -- C ABI of the mixed action+decode attention step over a shared, paged,
 * refcounted prefix KV cache (MI355X / gfx950).
 *
 * The paper's unified KV cache manager (Sec. 3.2; App. A.2) keeps one resumable
 * state per request, sigma = (KV cache, token buffer, termination flag), and
 * offers Store / Retrieve / Update / Remove plus Batch / UnBatch.  This library
 * is the KV part of that manager and the attention that reads it:
 *
 *   prefill cache K_t of a frame (Eq. 1)        -> a *prefix*: refcounted blocks, read-only
 *                                                  once anything is attached to it
 *   fan-out to action and language expert        -> *streams* attached to one prefix
 *   Store / Remove                               -> oxy_stream_create / oxy_stream_release
 *   Retrieve + Batch (Alg. 1, second stage)      -> oxy_batch_build (zero-copy: a descriptor
 *                                                  of block tables, no stacking of tensors)
 *   Update (KV grows by the decoded tokens)      -> oxy_batch_build (lengths, blocks) +
 *                                                  oxy_stream_append (the K/V rows)
 *   the attention of ActionDenoise / BatchedLanguageDecode (Eq. 5, Eq. 6)
 *                                                -> oxy_mixed_attention, one launch for
 *                                                  action-chunk and decode queries together
 *   UnBatch                                      -> nothing to do: block tables persist
 *
 * Geometry is fixed to the attention shape the kernels are written for:
 * 8 query heads sharing 1 KV head, head_dim 256, page size 16 tokens, bf16.
 *
 * Conventions
 *  - Every call returns 0 (OXY_OK) or a negative oxy_status; no C++ exception
 *    crosses this boundary.  oxy_last_error() gives a thread-local message.
 *  - A failing call changes no pool state (OXY_ERR_NO_BLOCKS is detected before
 *    any block is taken; a HIP launch or copy that fails inside oxy_prefix_append
 *    or oxy_batch_build gives its blocks and lengths back before returning).
 *  - Pointers marked DEVICE are device memory owned by the caller; pointers
 *    marked HOST are host memory owned by the caller.  The library owns only its
 *    host metadata and a small pinned staging buffer per live batch.
 *  - All device work is enqueued on the caller's hipStream_t (passed as void*);
 *    no call synchronises the device.  Calls that touch the same batch, or that
 *    free and re-use blocks, must be ordered on one HIP stream by the caller.
 *    A batch's descriptor and split results live in one of max_live_batches
 *    workspace slots, and oxy_batch_destroy hands the slot to the next
 *    oxy_batch_build at once, without waiting for the device: drive all batches of
 *    a pool on ONE HIP stream (then stream order protects the slot), or order the
 *    next build's stream behind the destroyed batch's last launch yourself.
 *  - Ids are sequential from 0 and never reused (App. A.2: the id of a request
 *    is the number of requests created before it); prefixes and streams count
 *    separately.
 *  - Not thread-safe per pool: one host thread drives one pool.
 *
 * Block pool policy (the paper has no allocator; this is the specification the
 * block tables are tested against, bit for bit): LIFO free stack whose initial
 * order is `free_order` (first element popped first; default 0,1,2,...); blocks
 * are popped one at a time in logical order, items of a batch in batch order;
 * release subtracts one reference per table entry and pushes, in ascending
 * logical order, the blocks that reach zero -- a stream's own table first, then
 * the table of the prefix it was attached to.
 *
 * Device layout of the KV buffer (private to the library, stated for the record):
 * layer l starts at l * num_blocks * 16 KiB; block b of a layer is 16 KiB: the
 * K page (8 KiB) then the V page (8 KiB).  Pages are stored in the operand
 * order of the 16x16x32 bf16 MFMA, so that every MFMA operand of the attention
 * kernel is one aligned 16-byte chunk:
 *   K page: chunk (j, hf, g, k8), j<8, hf<2, g<4, k8<8, at byte ((((j*2+hf)*4+g)*8)+k8)*16
 *           holds K[8hf+k8][32j+8g .. 32j+8g+7].
 *   V page: chunk (c, gp, m), c<16, gp<2, m<16, at byte (((c*2+gp)*16)+m)*16
 *           holds V[4gp..4gp+3][16c+m] followed by V[8+4gp..8+4gp+3][16c+m].
 * oxy_gather_kv reads tokens back in the natural [token][256] order.
 */
#ifndef OXY_H
#define OXY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  OXY_OK = 0,
  OXY_ERR_INVALID_ARG = -1, /* null pointer, size out of range, duplicate stream in a batch   */
  OXY_ERR_NO_BLOCKS = -2,   /* not enough free blocks; nothing was allocated                   */
  OXY_ERR_BAD_ID = -3,      /* unknown, released, or no longer attachable id                   */
  OXY_ERR_SEALED = -4,      /* append to a prefix that already has a stream attached           */
  OXY_ERR_BUSY = -5,        /* too many live batches, or pool destroyed with live batches      */
  OXY_ERR_WORKSPACE = -6,   /* batch does not fit the workspace the pool was created with      */
  OXY_ERR_DEVICE = -7       /* a HIP call failed; message holds hipGetErrorString              */
} oxy_status;

enum { OXY_KIND_ACTION = 0, OXY_KIND_DECODE = 1 };

/* pool flags */
enum { OXY_POOL_HOST_ONLY = 1 }; /* metadata only: no device pointer is touched, no HIP call is
                                    made; append/attention/gather return OXY_ERR_INVALID_ARG.
                                    For indexing tests on machines without a GPU.              */
/* batch flags */
enum { OXY_BATCH_APPEND_ONLY = 1 }; /* lengths, blocks and slots only; no attention work list
                                       (used to load a history); oxy_mixed_attention on such a
                                       batch returns OXY_ERR_INVALID_ARG                        */

typedef struct oxy_pool oxy_pool;   /* opaque host object                                   */
typedef struct oxy_batch oxy_batch; /* opaque; one step's descriptor (Alg. 1: the batched
                                       state, here block tables instead of stacked tensors) */

typedef struct {
  int32_t n_layers;         /* L >= 1                                                        */
  int32_t n_q_heads;        /* must be 8                                                     */
  int32_t n_kv_heads;       /* must be 1                                                     */
  int32_t head_dim;         /* must be 256                                                   */
  int32_t page_size;        /* must be 16                                                    */
  int32_t num_blocks;       /* capacity in blocks (one block = 16 tokens in every layer)     */
  void *kv_base;            /* DEVICE, >= oxy_kv_bytes(), 256-byte aligned                   */
  size_t kv_bytes;
  void *workspace;          /* DEVICE, >= oxy_workspace_bytes(), 256-byte aligned            */
  size_t workspace_bytes;
  const int32_t *free_order;/* HOST, optional permutation of [0,num_blocks); copied          */
  int32_t max_live_batches; /* descriptors that may exist at once (0 -> 2)                   */
  int32_t max_q_tokens;     /* query tokens per attended batch (0 -> 1024; at most 2^20)     */
  int32_t max_append_tokens;/* new tokens per batch, append-only ones included (0 -> 16*num_blocks) */
  int32_t max_work_items;   /* attention work items per batch (0 -> 16384)                   */
  int32_t max_partials;     /* per-token split results per batch (0 -> 32*max_q_tokens)      */
  int32_t split_tokens;     /* KV tokens per work item wherever query tokens share KV pages: the
                               prefix phase (tiles of 8 tokens on a prefix longer than 1024
                               tokens, streamed token pairs on a shorter one) and the own phase of
                               action chunks and multi-token decode.  Multiple of 32, <= 1024.
                               0 -> chosen from the length of the KV source alone: about an
                               eighth of it, within [64, 256]; 32 for a chunk of at most 64
                               tokens on an empty own history (an action chunk)             */
  int32_t stream_split_tokens; /* KV tokens per work item of the decode streaming path, multiple
                               of 32, <= 1024 (0 -> split_tokens; if that is 0 too: 128 for an own
                               history of at most 512 tokens, else 256).  Both depend
                               only on the pool and the item, so an item's arithmetic never
                               depends on its batch mates                                    */
  int32_t flags;
} oxy_pool_config;

typedef struct {
  int32_t stream_id;
  int32_t n_new; /* >= 1 tokens appended AND queried this step.  ACTION streams are rewound
                    to length 0 first: the chunk's K/V is transient per denoising step      */
} oxy_item;

/* sizes the caller must provide for kv_base / workspace (0 on invalid config) */
size_t oxy_kv_bytes(const oxy_pool_config *cfg);
size_t oxy_workspace_bytes(const oxy_pool_config *cfg);

/* Creates the host metadata; the KV buffer is not initialised (stale contents are never
 * read: keys beyond a length are masked and their values zero-selected). */
int32_t oxy_pool_create(const oxy_pool_config *cfg, oxy_pool **out);
int32_t oxy_pool_destroy(oxy_pool *pool); /* BUSY if batches are still alive */

/* --- prefix = prefill cache K_t of one observation (Sec. 3.1, Eq. 1) ------------------- */
int32_t oxy_prefix_create(oxy_pool *pool, int32_t *prefix_id); /* holds the creator's reference */
/* Writes tokens [pos0, pos0+n_tokens) of one layer.  k, v: DEVICE bf16 [n_tokens][256].
 * pos0 <= current length (no holes).  Blocks are taken the first time a token range is
 * reached (by whichever layer comes first).  SEALED once a stream is attached. */
int32_t oxy_prefix_append(oxy_pool *pool, int32_t prefix_id, int32_t layer, const void *k,
                          const void *v, int32_t n_tokens, int32_t pos0, void *hip_stream);
/* The same for layers [layer_begin, layer_end) in one call and one launch (the KV of a whole
 * prefill, Eq. 1): layer l reads k + (l - layer_begin) * layer_stride and v likewise (bytes). */
int32_t oxy_prefix_append_layers(oxy_pool *pool, int32_t prefix_id, int32_t layer_begin,
                                 int32_t layer_end, const void *k, const void *v,
                                 size_t layer_stride, int32_t n_tokens, int32_t pos0,
                                 void *hip_stream);
/* Fork (an extension for observations of consecutive frames that begin with the same history
 * segment): *prefix_id is a new prefix whose tokens 0..n_tokens-1 ARE the parent's — it lists the
 * parent's first n_tokens/16 blocks (refcount + 1 each, no copy).  n_tokens must be a multiple of
 * the page size and at most the parent's length; the caller must have appended that range in
 * every layer.  The shared range becomes read-only in parent and child (append below it:
 * OXY_ERR_SEALED); the child continues with oxy_prefix_append at pos0 >= n_tokens into blocks of
 * its own.  The parent may be any prefix that still exists, also one whose creator's reference
 * is gone but that requests keep alive. */
int32_t oxy_prefix_fork(oxy_pool *pool, int32_t parent_prefix_id, int32_t n_tokens,
                        int32_t *prefix_id);
/* Drops the creator's reference; attached streams keep the blocks alive (a request carried
 * over to later frames keeps the prefill cache of its birth frame, Sec. 3.2). */
int32_t oxy_prefix_release(oxy_pool *pool, int32_t prefix_id);

/* --- stream = KV part of one request state (Sec. 3.2, Eq. 3; App. A.2 Store/Remove) ---- */
int32_t oxy_stream_create(oxy_pool *pool, int32_t prefix_id /* -1: none */, int32_t kind,
                          int32_t *stream_id);
int32_t oxy_stream_release(oxy_pool *pool, int32_t stream_id);
int32_t oxy_stream_rewind(oxy_pool *pool, int32_t stream_id, int32_t new_len); /* keeps blocks */

/* --- one step (Alg. 1: Retrieve + Batch; App. A.2 Update) ------------------------------ */
/* items: HOST.  Extends every listed stream by n_new tokens (taking blocks as needed), records
 * the slot of every new token, builds the attention work list and uploads the descriptor on
 * hip_stream.  The descriptor serves every layer of the step. */
int32_t oxy_batch_build(oxy_pool *pool, const oxy_item *items, int32_t n_items, int32_t flags,
                        void *hip_stream, oxy_batch **out);
/* k_new, v_new: DEVICE bf16 [sum n_new][256], items in batch order.  Scatters them into the
 * slots of `layer`. */
int32_t oxy_stream_append(oxy_pool *pool, const oxy_batch *batch, int32_t layer,
                          const void *k_new, const void *v_new, void *hip_stream);
/* q: DEVICE bf16 [sum n_new][8][256]; out: DEVICE bf16, same shape; lse: DEVICE float
 * [sum n_new][8] or NULL (natural-log sum of exp of the scaled logits over the visible set).
 * Visible set of a query (Eq. 2, Eq. 5, Eq. 6): the whole prefix of its stream, plus
 *   ACTION: every own token of the chunk (bidirectional);
 *   DECODE: own tokens 0..p where p is the query's own position (causal, itself included).
 * Must be enqueued after oxy_stream_append of the same layer on the same stream. */
int32_t oxy_mixed_attention(oxy_pool *pool, const oxy_batch *batch, int32_t layer,
                            const void *q, void *out, float *lse, float scale,
                            void *hip_stream);
/* oxy_mixed_attention for callers that cannot allocate device memory or hand a workspace of
 * matching size to the call: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels, same outputs; the per-split results
 * (un-normalised accumulators and softmax statistics, which oxy_mixed_attention keeps in the
 * batch's workspace slot) live in a static device array inside the library instead: 2048 split
 * results (8.25 MiB), held by every GPU the library runs on until the process ends.  The call
 * allocates nothing and frees nothing.  OXY_ERR_WORKSPACE if the batch has more than 2048
 * split results (oxy_batch_info: n_partials).  Every call on a GPU uses that GPU's one array:
 * calls that overlap on one GPU (different HIP streams, or the same batch on two streams)
 * race; calls ordered on one stream do not, and nothing in the array needs clearing between
 * calls (every entry a launch reads was written by that launch). */
int32_t oxy_mixed_attention_static(oxy_pool *pool, const oxy_batch *batch, int32_t layer,
                                   const void *q, void *out, float *lse, float scale,
                                   void *hip_stream);
/* All layers [layer_begin, layer_end) of one step, in order: for each layer the append and
 * then the mixed attention, with the same kernels and the same effects as the two calls above
 * (this is their loop moved below the ABI: one call per step instead of two per layer).
 * Layer l uses k_new + l*kv_layer_stride, v_new + l*kv_layer_stride (bytes), q + l*q_layer_stride,
 * out + l*q_layer_stride, and lse + l*lse_layer_stride (bytes) when lse is not NULL.
 * flags: 0 = three launches per layer (append, work items, merge), the order a model imposes
 * when layer l+1's K/V depend on layer l's output.  OXY_STEP_FUSE_ACROSS_LAYERS = the merge of
 * layer l shares its launch with the append of layer l+1 (disjoint memory); only meaningful when
 * every layer's new K/V is known up front (attention-only replay, benchmarking).
 * OXY_STEP_FOLD_APPEND = the work items themselves write the new rows (two launches per layer):
 * a decode item's new token is read only by the work item that owns the last split of its own
 * history, so that work item writes it first; an item whose own history was empty before the
 * step (an action chunk, Sec. 3.2: its K/V live for one denoise step) reads its keys from
 * k_new / v_new directly (the layer's merge launch writes them to the pool).  Outputs and pool contents
 * are those of flags = 0.  A batch with an item of more than 2 new tokens on a non-empty own
 * history is not covered; for it the flag is ignored.  Wins over OXY_STEP_FUSE_ACROSS_LAYERS.
 * OXY_STEP_GRAPH (with any of the above) = the launches of the step are recorded into a HIP graph
 * the first time a step of this form is seen and replayed with ONE graph launch on hip_stream
 * from then on: Alg. 1's S denoise steps and k decode steps per frame are short launches, and
 * issuing 2-3 of them per layer from the host costs more than running them.  "This form" = same
 * workspace slot, same pointers, strides, scale and layers, same numbers of tokens and work
 * items; a decode loop with resident buffers meets this on every step until a history crosses a
 * split boundary.  A step of a new form is recorded again (an existing recording with the same
 * launch sequence is updated in place once eight are held).  Same kernels, same arguments,
 * same results bit for bit.  The pool keeps the recordings until it is destroyed; the pointers
 * must stay valid while steps of that form are replayed.  events must be NULL.
 * events: NULL, or HOST array of 4*(layer_end-layer_begin) entries, each a created hipEvent_t or
 * NULL; per layer they receive the begin and end timestamps of the work-item kernel and of the
 * merge kernel themselves (hipExtLaunchKernel start/stop events; a profiling hook).  A launch
 * whose two entries are NULL is issued exactly as without events. */
enum { OXY_STEP_FUSE_ACROSS_LAYERS = 1, OXY_STEP_FOLD_APPEND = 2, OXY_STEP_GRAPH = 4 };
int32_t oxy_step_layers(oxy_pool *pool, const oxy_batch *batch, int32_t layer_begin,
                        int32_t layer_end, const void *k_new, const void *v_new,
                        size_t kv_layer_stride, const void *q, void *out, size_t q_layer_stride,
                        float *lse, size_t lse_layer_stride, float scale, int32_t flags,
                        void *const *events, void *hip_stream);
/* Counters of OXY_STEP_GRAPH since the pool was created (any output may be NULL): recordings
 * instantiated, recordings updated in place, steps replayed. */
int32_t oxy_step_graph_stats(oxy_pool *pool, int32_t *instantiations, int32_t *updates,
                             int32_t *replays);
/* oxy_stream_append + oxy_mixed_attention of one layer in two launches instead of three: the
 * KV part of Update (App. A.2) folded into the attention work items, see OXY_STEP_FOLD_APPEND.
 * k_new, v_new: DEVICE bf16 [n_tokens][256] of this layer; q, out, lse as oxy_mixed_attention. */
int32_t oxy_append_attention(oxy_pool *pool, const oxy_batch *batch, int32_t layer,
                             const void *k_new, const void *v_new, const void *q, void *out,
                             float *lse, float scale, void *hip_stream);
int32_t oxy_batch_destroy(oxy_batch *batch);

/* Reads K/V rows back in natural order: slots HOST int64 [n] (block*16+offset);
 * k_out, v_out: DEVICE bf16 [n][256]. */
int32_t oxy_gather_kv(oxy_pool *pool, int32_t layer, const int64_t *slots, int32_t n,
                      void *k_out, void *v_out, void *hip_stream);

/* --- introspection (HOST outputs; these are the indexing results compared bit-exactly) -- */
int32_t oxy_stream_info(oxy_pool *pool, int32_t stream_id, int32_t *prefix_id, int32_t *kind,
                        int32_t *own_len, int32_t *n_blocks);
int32_t oxy_stream_blocks(oxy_pool *pool, int32_t stream_id, int32_t *out, int32_t cap);
int32_t oxy_prefix_info(oxy_pool *pool, int32_t prefix_id, int32_t *len, int32_t *n_blocks,
                        int32_t *sealed, int32_t *n_streams);
int32_t oxy_prefix_blocks(oxy_pool *pool, int32_t prefix_id, int32_t *out, int32_t cap);
int32_t oxy_block_refcounts(oxy_pool *pool, int32_t *out, int32_t cap); /* cap >= num_blocks */
int32_t oxy_free_blocks(oxy_pool *pool, int32_t *out, int32_t cap);     /* top of stack first */
int32_t oxy_pool_stats(oxy_pool *pool, int32_t *free_blocks, int32_t *live_prefixes,
                       int32_t *live_streams);
int32_t oxy_batch_info(const oxy_batch *batch, int32_t *n_items, int32_t *n_tokens,
                       int32_t *n_work, int32_t *n_partials);
int32_t oxy_batch_slots(const oxy_batch *batch, int64_t *out, int32_t cap);
/* Raw work list, 8 int32 per item: token-list offset, token count, block-table offset,
 * kv_begin, kv_end, causal base position (or 0x3fffffff), partial index, path. */
int32_t oxy_batch_work(const oxy_batch *batch, int32_t *out, int32_t cap_items);

/* --- frame scheduler: the per-frame execution flow (Alg. 1, App. A.3; Sec. 3.2) --------
 * Host logic only.  Per frame: the caller appends the prefill KV of each new observation to a
 * fresh prefix and admits it; the scheduler fans it out (Alg. 1 lines 2-5: an ACTION stream that
 * is denoised over S steps, and a DECODE stream = a new language request under the next
 * request id, App. A.2), then hands out the frame's steps one by one (lines 6-9): step s lists
 * the chunk of every observation admitted in this frame while s < S and one token for every
 * active request that has neither finished nor used up the per-frame budget k; the caller runs
 * each step (oxy_batch_build, then append + attention per layer).  oxy_sched_end_frame evicts the
 * finished requests and persists the rest (lines 10-13).  Any number of observations may
 * arrive in a frame, also none (Sec. 4.4).  Termination is by length only (no logits here).
 * mode (Sec. 4.3): OXY_SCHED_BATCHED = the flow above; OXY_SCHED_UNBATCHED = cross-task sharing
 * without cross-frame batching: observations are served one after the other and each request
 * runs to completion inside its frame; OXY_SCHED_UPPER_BOUND = the single-frame decoding oracle
 * of the ablation: k tokens, then the request is dropped at frame end.
 * Items of a step: action chunks in admission order, then requests in ascending id. */
typedef struct oxy_sched oxy_sched;
enum { OXY_SCHED_BATCHED = 0, OXY_SCHED_UNBATCHED = 1, OXY_SCHED_UPPER_BOUND = 2 };
typedef struct {
  int32_t k;             /* decode steps per request per frame (Alg. 1 input k), >= 1 */
  int32_t denoise_steps; /* S; 0 = no action expert (then chunk must be 0 too) */
  int32_t chunk;         /* action tokens per denoise step (H) */
  int32_t max_active;    /* capacity of the active set R; 0 = unbounded.  An observation that
                            arrives while R is full still gets its action, but no request */
  int32_t mode;
} oxy_sched_config;
int32_t oxy_sched_create(oxy_pool *pool, const oxy_sched_config *cfg, oxy_sched **out);
/* Releases every stream the scheduler still holds and the prefixes of an unfinished frame. */
int32_t oxy_sched_destroy(oxy_sched *sched);
/* One new observation whose prefill KV is prefix_id (appended by the caller, all layers); only
 * before the first step of a frame.  target_len = N, the request's total decode length.
 * *request_id = the new id, or -1 if the active set is full.  The scheduler takes over the
 * creator's reference of the prefix and drops it at the end of the frame. */
int32_t oxy_sched_admit(oxy_sched *sched, int32_t prefix_id, int32_t target_len,
                        int32_t *request_id);
/* The next step of the current frame: items HOST [cap] receives *n_items (stream, n_new) pairs
 * ready for oxy_batch_build, of which the first *n_action_items (may be NULL) are action
 * chunks.  *n_items = 0: the frame has no more steps.  A returned step counts as executed. */
int32_t oxy_sched_next_step(oxy_sched *sched, oxy_item *items, int32_t cap, int32_t *n_items,
                            int32_t *n_action_items);
/* Only when the frame has no more steps.  Releases the frame's action streams, the finished
 * requests (ascending id, written to finished HOST [cap]) and the frame's prefixes. */
int32_t oxy_sched_end_frame(oxy_sched *sched, int32_t *finished, int32_t cap,
                            int32_t *n_finished);
/* Offline calibration of the per-frame budget k (Sec. 3.2): the largest k in 1..target_len whose
 * steady-state frame, with arrivals_per_frame observations arriving in every frame, fits into
 * frame_budget (= 1 / target frame rate).  The caller measures the costs, all in one unit of
 * time: t_observation per arriving observation (prefill and fan-out), t_mixed[b] for a step
 * that denoises while b requests decode, t_decode[b] for a decode-only step with b requests
 * (HOST arrays of n_table entries, index b; t_decode[0] is never read).  *k_out = 0 if no k
 * meets the budget; *frame_time_out (may be NULL) = the modelled frame time at *k_out.
 * OXY_ERR_INVALID_ARG if a batch size that occurs is not covered by the tables. */
int32_t oxy_sched_calibrate(const double *t_mixed, const double *t_decode, int32_t n_table,
                            double t_observation, int32_t denoise_steps, int32_t target_len,
                            int32_t arrivals_per_frame, double frame_budget, int32_t *k_out,
                            double *frame_time_out);
int32_t oxy_sched_info(oxy_sched *sched, int32_t *frame, int32_t *n_active, int32_t *n_created,
                       int32_t *n_rejected);
/* OXY_ERR_BAD_ID if the request is not in the active set (any output may be NULL). */
int32_t oxy_sched_request_info(oxy_sched *sched, int32_t request_id, int32_t *stream_id,
                               int32_t *done, int32_t *target, int32_t *birth_frame);

const char *oxy_last_error(void);
int32_t oxy_version(void);

#ifdef __cplusplus
}
#endif
#endif /* OXY_H */
