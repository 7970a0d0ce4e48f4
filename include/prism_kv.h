/*
 * prism_kv.h — C-ABI boundary of the MI355X (gfx950) shared-pool paged decode
 * attention library (libprismkv.so).
 *
 * The library is the hot path behind GPU memory ballooning for multi-LLM
 * co-serving: several co-located models keep their KV cache in ONE physical page
 * pool; each model's share of the pool (its balloon) grows and shrinks between
 * decode steps; decode attention reads K and V through per-sequence block tables.
 *
 * Vocabulary
 *   frame   fixed-size physical unit of the pool (the paper's 2 MB physical page,
 *           Sec. 4.2 D3).  Owned by at most one model (D2: models never share a
 *           page).  balloon_resize counts frames.
 *   block   page_tokens tokens of one model's K and V for all its KV heads (the
 *           paper's token block / KV block, Background "KV cache and
 *           PagedAttention").  block_bytes = 2*page_tokens*kv_heads*head_dim*e,
 *           e = 2 for bf16 and 1 for e4m3, plus a 128-byte scale header for e4m3.
 *           A model registered with several layers keeps all of them in the block
 *           (n_layers times those bytes, see model_register_layers).
 *   slot    place for one block inside a frame; slots = frame_bytes / block_bytes.
 *   block id = frame * slots + slot  (what block tables hold).
 *
 * Conventions
 *   - Every function returns 0 or a non-negative count on success and a negative
 *     PKV_E_* code on error.  Nothing throws or aborts.  A failing call leaves the
 *     bookkeeping state unchanged (balloon deflate clamps instead of failing).
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host
 *     addresses.  Unless stated, buffers belong to the caller.
 *   - Work is enqueued on the HIP stream given to pkv_set_stream (default: the
 *     null stream).  Bookkeeping calls that return a count wait for their kernel
 *     (their *_enqueue forms do not); kv_write and the decode_attention family only enqueue.
 *   - All bookkeeping (free stack, ownership, frame lists, slot bitmaps, block
 *     tables) lives in device memory and is changed only by the library's kernels.
 *   - Calls are not thread-safe; one thread drives one library instance.
 *   - Streams: a call enqueues on the stream that was current when it was made.  The
 *     bookkeeping calls of one pool must all go to one stream (or be ordered by the
 *     caller); attention and KV calls may go to other streams once the caller has ordered
 *     them behind the bookkeeping they depend on.  A model has ONE split-K workspace: two
 *     decode_attention* calls on the same model must not overlap in time (different models
 *     may).  The workspace is sized when the model is registered, so decode_attention*
 *     neither allocates nor waits and can be captured into a HIP graph without a priming
 *     launch; the exceptions are a caller's block table with more rows than the model was
 *     registered for, and a work-item count raised through the tuning header.
 *   - Knobs and probes for measurements and tests live in prism_kv_tuning.h.
 */
#ifndef PRISM_KV_H
#define PRISM_KV_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    PKV_OK = 0,
    PKV_E_ARG = -1,         /* bad argument value */
    PKV_E_HANDLE = -2,      /* unknown pool / model id */
    PKV_E_NOMEM = -3,       /* inflate: not enough free frames; or no id / memory left */
    PKV_E_BALLOON = -4,     /* reserve: not enough free slots in the model's balloon */
    PKV_E_SHAPE = -5,       /* block does not fit a frame, q_heads % kv_heads != 0 */
    PKV_E_RANGE = -6,       /* index outside a table / buffer too small */
    PKV_E_BUSY = -7,        /* destroy / unregister while frames are still owned */
    PKV_E_INTERNAL = -8,
    PKV_E_DEVICE = -9,      /* a HIP call failed; see pkv_last_error() */
    PKV_E_UNSUPPORTED = -10 /* shape the gfx950 kernels do not cover */
};

enum { PKV_BF16 = 0, PKV_E4M3 = 1 };

typedef struct pkv_stats {
    int64_t n_frames, n_free;   /* pool */
    int64_t owned[64];          /* frames per model id (0 for ids not in this pool) */
    int64_t used_blocks[64];    /* reserved blocks per model id */
    int64_t mapped_bytes;       /* pool bytes backed by device memory (all of it unless the pool is elastic) */
    int64_t spare_frames;       /* (always 0: kept for the layout of the structure) */
    int64_t idle_frames;        /* elastic pools: frames that have memory but no owner (the pre-allocation buffer) */
} pkv_stats;

/* ---- library ------------------------------------------------------------ */

/* Select the HIP stream (a hipStream_t, e.g. torch.cuda.current_stream().cuda_stream)
 * all later calls enqueue on.  NULL = the null stream. */
int pkv_set_stream(void *hip_stream);
/* Text of the last HIP / library error on this thread (never NULL). */
const char *pkv_last_error(void);
/* Sticky device-side error flags raised by calls that only enqueue (bit 0: a block id outside
 * the pool was met in decode_attention, that page was skipped; bit 1: kv_append met a context
 * length outside the row's blocks; bit 2: an enqueue-only bookkeeping call was refused).
 * Synchronises the stream; clears the flags. */
int pkv_device_errors(void);

/* ---- pool (paper Sec. 4.2: one physical pool for all co-located models) -- */

/* Create a pool of `bytes` bytes cut into 2 MiB frames (D3: 2 MB pages);
 * page_tokens = tokens per block.  The library allocates the device memory.
 * Returns the pool id (lowest unused, 0..7).  The free stack starts so that
 * frames are handed out in the order 0, 1, 2, ... */
int pool_create(size_t bytes, int page_tokens);
/* Same with an explicit frame size and optionally caller-owned device memory
 * (device_base, dev, at least bytes long, 256-byte aligned; NULL = allocate). */
int pool_create_ex(size_t bytes, int page_tokens, size_t frame_bytes, void *device_base);
/* A pool whose memory is elastic (paper Sec. 4.2, D1 / D3: the balloon driver hands physical
 * pages out lazily and takes them back, so that what one model gives up can serve another
 * model or its weights).  The pool is a reserved range of device addresses; a frame is backed
 * by device memory while a model owns it (HIP virtual memory management), and besides that only
 * while it waits in the pre-allocation buffer.  frame_bytes must be a multiple of the device's
 * allocation granularity (PKV_E_SHAPE).  Everything else behaves like pool_create_ex;
 * pool_stats reports mapped_bytes and idle_frames (frames that have memory but no owner).
 *
 * The pre-allocation buffer (paper D3: a pre-allocation thread keeps pages ready so that the
 * cost of mapping stays off the critical path): pool_set_prealloc(pool, n) asks that the n
 * frames on top of the free stack — the next n an inflate will be given — have memory.  An
 * inflate of up to n frames then maps nothing, and no balloon_resize ever unmaps: a deflate
 * pushes its frames, memory and all, on top of the stack and returns.  A thread of the
 * library restores the rule afterwards: it creates and maps memory for frames that have risen
 * into the top n, and unmaps and releases the free frames that have sunk below them (about
 * 50 us per frame to map, 250 us to unmap, so mapped_bytes is back at (owned + n) frames within
 * roughly 0.3 ms per frame moved).  An inflate that outruns the thread maps what is missing
 * itself, as it does for everything beyond n.  pool_set_prealloc waits until the buffer
 * stands and returns the frames held; pool_prealloc_wait waits until the thread has caught up
 * with every balloon_resize so far and returns the same.  n = 0 (the start) keeps nothing. */
int pool_create_elastic(size_t bytes, int page_tokens, size_t frame_bytes);
int pool_set_prealloc(int pool, long frames);
int pool_prealloc_wait(int pool);
/* Fails with PKV_E_BUSY while any model is registered in the pool. */
int pool_destroy(int pool);
/* Set the order in which a still-untouched pool hands out frames: perm (host,
 * n = number of frames) is a permutation of the frame ids, perm[0] first. */
int pool_seed_free_order(int pool, const uint32_t *perm, size_t n);

/* ---- models (D2: automatic token-block mapping, per-model segregation) --- */

/* Register a model in the most recently created pool, with room for 256
 * sequences of up to 2048 blocks.  dtype = PKV_BF16 | PKV_E4M3 (KV storage;
 * queries are always bf16).  Returns the model id (lowest unused, 0..63). */
int model_register(int q_heads, int kv_heads, int head_dim, int dtype);
int model_register_ex(int pool, int q_heads, int kv_heads, int head_dim, int dtype,
                      int max_seqs, int max_blocks_per_seq);
/* A model of n_layers layers (paper Sec. 4.2, D3, first optimisation: the K and V of all
 * layers of a token block lie side by side, so one allocation serves every layer instead of
 * 2L).  A block is n_layers consecutive one-layer blocks (each laid out as for a one-layer
 * model, the e4m3 header included); block ids, slots, the block table and every bookkeeping
 * call are shared by the layers, frames hold frame_bytes / (n_layers * layer bytes) blocks
 * (PKV_E_SHAPE if that is zero).  pkv_set_layer picks the layer (0 at registration) that
 * kv_write, kv_append, kv_append_chunk, kv_read, decode_attention, decode_attention_multi
 * and prefill_attention address from then on; it is host state only (no device work,
 * PKV_E_ARG outside 0..n_layers-1) and takes effect for calls enqueued after it. */
int model_register_layers(int pool, int q_heads, int kv_heads, int head_dim, int dtype,
                          int max_seqs, int max_blocks_per_seq, int n_layers);
int pkv_set_layer(int model, int layer);
/* The model must own no frames (PKV_E_BUSY otherwise). */
int model_unregister(int model);

/* ---- balloon (D1: per-model limits that shrink and grow) ------------------ */

/* Make the model own `pages` frames.
 *   inflate: frames are popped from the pool's free stack and appended to the
 *            model's frame list; PKV_E_NOMEM if the pool has too few (no change), or
 *            if an elastic pool gets no memory for one of them (the inflate is undone:
 *            no change either).
 *   deflate: empty frames are returned to the free stack, newest first, until
 *            the target is met; frames that still hold blocks stay.
 * Returns the number of frames owned afterwards (>= pages on a clamped deflate). */
long balloon_resize(int model, long pages);

/* Grow sequence `seq`'s block-table row to ceil(ctx_len / page_tokens) blocks,
 * taking the lowest free slots of the model's frames in frame-list order.
 * Returns the number of blocks added; PKV_E_BALLOON if the balloon has too few
 * free slots (no change); PKV_E_RANGE beyond max_blocks_per_seq. */
int seq_reserve(int model, int seq, int ctx_len);
/* Same effect as seq_reserve for (seqs[i], ctx_lens[i]), i = 0..n-1 in order, in
 * one kernel launch; refused as a whole when the total does not fit.  A sequence may be
 * listed more than once (the growth rounds of a whole admission in one call).
 * seqs, ctx_lens: host, n <= 4096. */
int seq_reserve_batch(int model, int n, const int32_t *seqs, const int32_t *ctx_lens);
/* Free all blocks of the row; returns how many (0 for an empty row). */
int seq_release(int model, int seq);
/* Same effect as seq_release for seqs[0..n-1] in order, in one kernel launch; returns the
 * blocks freed in total.  seqs: host, n <= 4096. */
int seq_release_batch(int model, int n, const int32_t *seqs);

/* ---- the same bookkeeping, enqueue-only ------------------------------------------------------
 * A serving loop issues the bookkeeping of a step (the deflates of models that fell idle, the
 * inflate and the reservations of an admission: Sec. 3.1 bursty groups, Sec. 4.2 D1 / D2) and
 * goes on to enqueue the step's attention without waiting for any of it.  These forms launch the
 * same kernels as balloon_resize, seq_reserve_batch and seq_release_batch, in stream order, and
 * return at once with a ticket (>= 0) instead of the result; argument errors that need no device
 * state still come back at once as a negative code (unknown model, bad n, NULL list).
 *   - pkv_ticket_result(ticket) waits for that call if need be and returns what the synchronous
 *     form would have returned.  The library remembers the last 128 tickets (PKV_E_RANGE for an
 *     older one).
 *   - A refused call (PKV_E_NOMEM, PKV_E_BALLOON, PKV_E_ARG, PKV_E_RANGE) changes nothing, as in
 *     the synchronous form, and raises bit 2 of pkv_device_errors(), so a caller need not read
 *     every ticket.  Later calls run against the unchanged state: a reserve after a refused
 *     inflate is refused too, and attention over rows that never got their blocks reads nothing
 *     (the kernels bound every row by the blocks it really holds).
 *   - All bookkeeping calls of a pool must go to one stream, or be ordered by the caller.
 *   - On an elastic pool balloon_resize_enqueue does its work at once (mapping frames is host
 *     work) and returns a ticket that is already complete. */
int balloon_resize_enqueue(int model, long pages);
int seq_reserve_batch_enqueue(int model, int n, const int32_t *seqs, const int32_t *ctx_lens);
int seq_release_batch_enqueue(int model, int n, const int32_t *seqs);
long pkv_ticket_result(int ticket);

/* Device pointer to the model's block table, int32 [max_seqs][*row_stride],
 * owned by the library, valid until model_unregister. */
const int32_t *model_block_table(int model, int *row_stride);

/* ---- KV data -------------------------------------------------------------- */

/* Scatter tokens [tok_begin, tok_begin + n_tok) of sequence `seq` from logical
 * layout into its reserved blocks.  k, v: dev, [n_tok][kv_heads][head_dim] bf16
 * values or e4m3 codes.  e4m3 only: k_scale, v_scale: dev, fp32
 * [blocks touched][kv_heads], row 0 = the block holding tok_begin; the value of an
 * element is decode(code) * scale.  Enqueues only. */
int kv_write(int model, int seq, int tok_begin, int n_tok, const void *k, const void *v,
             const float *k_scale, const float *v_scale);

/* The write path of a decode step (paper Sec. 4.2, D2: a growing sequence takes its next
 * token block from the slots of its pages): for every sequence s < batch the token with
 * index ctx_lens[s] - 1 is written into the row's reserved blocks (the library's table).
 * k_new, v_new: dev, bf16 [batch][kv_heads][head_dim], the values as the model produced
 * them, for both cache types.  ctx_lens: dev int32 [batch].
 * e4m3 models quantise here, one fp32 scale per (block, kv head) for K and for V, kept
 * equal to the running maximum of amax / 448 over the block's tokens (fp32 arithmetic,
 * round to nearest even, saturating):  slot 0 of a block: scale = amax > 0 ? amax/448 : 1;
 * later slots: cand = amax/448, and if cand > scale every code c already in the block
 * becomes encode((decode(c) * scale) / cand) and scale = cand;  the new token's codes are
 * encode(x / scale).
 * A context length outside 1 .. 16 * (blocks reserved for the row) is skipped and sets
 * bit 1 of pkv_device_errors().  Returns batch; PKV_E_RANGE if batch exceeds the model's
 * rows.  Enqueues only. */
int kv_append(int model, int batch, const void *k_new, const void *v_new, const int32_t *ctx_lens);

/* The write path of a prefill chunk: sequence s < batch appends its q_lens[s] new tokens,
 * packed one sequence after the other in k_new, v_new (dev, bf16 [sum q_lens][kv_heads]
 * [head_dim]), at the indices ctx_lens[s] - q_lens[s] .. ctx_lens[s] - 1.  The result is that
 * of kv_append applied token by token in order (so a cache filled in chunks equals one
 * filled a token at a time, e4m3 codes and scales included).  q_lens: HOST int32 [batch];
 * ctx_lens: dev int32 [batch].  Returns sum q_lens.  Enqueues only (plus a small
 * host-to-device copy of the chunk list); errors as kv_append. */
int kv_append_chunk(int model, int batch, const void *k_new, const void *v_new, const int32_t *q_lens,
                    const int32_t *ctx_lens);

/* Tokens [tok_begin, tok_begin + n_tok) of a sequence back in the logical layout of
 * kv_write: k_out, v_out dev [n_tok][kv_heads][head_dim] (bf16 values or e4m3 codes);
 * e4m3 only: k_scale_out, v_scale_out dev fp32 [n_tok][kv_heads], the scale of the
 * block each token lives in.  For tests and debugging.  Enqueues only. */
int kv_read(int model, int seq, int tok_begin, int n_tok, void *k_out, void *v_out,
            float *k_scale_out, float *v_scale_out);

/* ---- decode attention (Background: paged attention over the block table) -- */

/* Batch shape used by decode_attention: `batch` sequences, caller block tables
 * with `row_stride` int32 entries per row. */
int model_set_batch(int model, int batch, int row_stride);

/* out[s][h][:] = softmax_t( q[s][h] . K[t][h/g] / sqrt(head_dim) ) V[t][h/g][:]
 * over t < ctx_lens[s], g = q_heads / kv_heads, K/V read through the block table.
 *   q           dev, bf16 [batch][q_heads][head_dim]
 *   block_table dev, int32 [batch][row_stride] block ids; NULL = the library's own
 *               table, rows 0..batch-1.  A caller's table is refused on an elastic pool
 *               (PKV_E_UNSUPPORTED): its ids could name frames that nothing backs.
 *   ctx_lens    dev, int32 [batch]; 0 gives a zero output row
 *   out         dev, fp32 [batch][q_heads][head_dim]
 * fp32 accumulation.  Enqueues only. */
int decode_attention(int model, const void *q, const int32_t *block_table,
                     const int32_t *ctx_lens, float *out);
int decode_attention_ex(int model, int batch, const void *q, const int32_t *block_table,
                        int row_stride, const int32_t *ctx_lens, float *out);
/* decode_attention_ex for callers that cannot allocate device memory or wait for the stream:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same result (up to the rounding of a different split), every cache type, but the
 * split-K partials and arrival counters of its kernel live in a 20 MiB array that is part of
 * the library's device code (one copy per GPU, held until the process ends) instead of the
 * model's workspace.  The call allocates nothing, frees nothing and never waits; it enqueues
 * a small kernel that clears the counters it needs, then the attention kernel.
 * Limits: batch * kv_heads <= 32768 (PKV_E_RANGE, with a message in pkv_last_error()); when
 * the partials of the usual number of work items do not fit the array, fewer items are used.
 * All calls on one GPU share the one array: two such calls must not overlap in time (on
 * different streams, or from different threads) — the second would clear counters the first
 * still uses. */
int decode_attention_static(int model, int batch, const void *q, const int32_t *block_table,
                            int row_stride, const int32_t *ctx_lens, float *out);
/* One grouped launch over several models of one pool (the multi-model decode
 * step); each uses the library's own block table rows 0..batches[i]-1.
 * models, batches, q, ctx_lens, out: host arrays of n_models entries holding
 * ids / sizes / dev pointers. */
int decode_attention_multi(int n_models, const int *models, const int *batches,
                           const void *const *q, const int32_t *const *ctx_lens,
                           float *const *out);

/* Causal attention of prefill chunks against the paged cache (paper Sec. 5.2: prefill runs
 * in chunks, each attending to the cache built so far).  Sequence s < batch brings
 * q_lens[s] new query tokens, packed one sequence after the other in q (dev, bf16
 * [sum q_lens][q_heads][head_dim]); its cache holds ctx_lens[s] tokens, the chunk's own
 * included (write them first: kv_write or kv_append).  Query i of the sequence stands at
 * position ctx_lens[s] - q_lens[s] + i and sees the tokens at or before it:
 *     out = softmax over t <= position of (q . k[t] / sqrt(head_dim)) V
 * out: dev fp32 [sum q_lens][q_heads][head_dim].  q_lens: HOST int32 [batch] (the caller's
 * scheduler chose the chunk sizes); ctx_lens: dev int32 [batch].  The library's table is
 * used.  A sequence whose ctx_lens is below its q_lens gets zero rows for the queries
 * that would stand before position 0.  Enqueues only (a small host-to-device copy of the
 * row plan included); a call with few query tokens in front of long contexts splits the
 * contexts over several work-groups and then keeps partial results in a per-model buffer
 * that the library allocates, or enlarges after waiting for the stream, when it is first
 * needed. */
int prefill_attention(int model, int batch, const void *q, const int32_t *q_lens,
                      const int32_t *ctx_lens, float *out);

/* ---- observation ----------------------------------------------------------- */

/* Canonical image of the bookkeeping state as little-endian int32 words:
 *   "PKVS", version 1, n_frames, page_tokens, n_free, free stack bottom..top,
 *   owner[n_frames] (-1 = free), n_models, then per model in id order:
 *   id, q_heads, kv_heads, head_dim, dtype, slots, owned, frames[owned], nbits,
 *   ceil(nbits/32) words of slot bits (bit j = slot j%slots of frame j/slots),
 *   max_seqs, n_rows, then per non-empty row: seq, len, block ids.
 * host_buf: host.  Returns the byte size needed; writes only if cap suffices.
 * Synchronises the stream. */
long pool_export_state(int pool, void *host_buf, size_t cap);
int pool_stats(int pool, pkv_stats *out);

/* ---- policies that drive the balloons (host only; no stream, no device) ---------------- */

/* Slack-aware request arbitration on one GPU (paper Sec. 5.2, Alg. 2: the Moore-Hodgson rule on
 * prefill deadlines).  Request i waits since arrival[i], must finish its prefill by arrival[i] +
 * ttft_slo[i], and its prefill takes prompt_len[i] / prefill_speed[i].  Requests are taken in
 * order of deadline (equal deadlines: lower index first), appended to the schedule S, and
 * whenever the newcomer would finish after its deadline the request of S with the longest
 * prefill is dropped (equal lengths: the one earliest in S).  accepted (out, int32 [n], host)
 * receives the indices of S in dispatch order; returns their number, which is the largest
 * number of requests that can all meet their deadlines.  All arrays are host arrays. */
int arbitrate_requests(int n, const double *arrival, const double *ttft_slo, const double *prompt_len,
                       const double *prefill_speed, double now, int32_t *accepted);

/* Model placement by KV pressure ratio (paper Sec. 5.1, Alg. 1).  Model j asks for memory at
 * the SLO-weighted rate token_rate[j] * token_size[j] / slo[j] and occupies weight[j] bytes; a
 * GPU's KV pressure ratio is the summed rate of its models over capacity minus their weights
 * (infinite once nothing is left).  Models are taken by falling rate (equal: lower index
 * first); each goes to the GPU of lowest ratio (equal: lower index) unless it already sits on
 * a GPU (current_gpu[j] >= 0) whose ratio is not more than tau above that: then it stays.
 * tp_group (NULL or int32 [n_models]): models with the same id >= 0 are parts of one
 * tensor-parallel model and never share a GPU (PKV_E_RANGE if there are more parts than GPUs);
 * the caller splits weight and rate among the parts.  gpu_out (int32 [n_models]) receives the
 * placement; returns n_models.  All arrays are host arrays; current_gpu may be NULL. */
int place_models(int n_gpus, double capacity, double tau, int n_models, const double *token_rate,
                 const double *token_size, const double *slo, const double *weight,
                 const int32_t *current_gpu, const int32_t *tp_group, int32_t *gpu_out);

#ifdef __cplusplus
}
#endif
#endif
