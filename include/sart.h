/*
 * sart.h - C ABI of the SART branch-serving hot path for AMD MI355X (gfx950).
 *
 * The paper (arXiv 2505.13326) schedules N sampled reasoning branches per
 * request, decodes them in one batch, and removes branches from the batch when
 * they complete, are pruned by a reward threshold, or are early-stopped once
 * enough branches of the request completed (Algorithm 1, functions Prefill and
 * Decode).  Section 4 (its paragraph on KV-cache management) fixes the
 * KV-cache rule this library implements: the prompt's KV cache is shared by
 * all branches of a request, a branch's own KV cache is released immediately
 * when it is pruned, early-stopped or completed, and the shared prefix is
 * released only when every branch of the request has terminated.
 *
 * Everything below is device resident: the paged KV pool, the free-page stack,
 * the per-request prefix tables, the per-branch block tables and the active
 * list live in HBM and are only changed by kernels.  Calls enqueue work on the
 * caller's HIP stream and return; only sart_get_state and sart_sync_status
 * wait for the device.
 *
 * Vocabulary
 *   Nb      branches sampled per request (the paper's N).
 *   Q       completions that trigger early stop (the paper's M).
 *   handle  r*Nb + j, the j-th branch of request r; stable for life.
 *   active index  row of a branch in the compacted active list.  Rows of q,
 *           out and scores are in active order.
 *   page    page_tokens consecutive tokens of one sequence, all KV heads.
 *
 * Pointers are marked HOST or DEVICE.  The library never keeps a caller
 * pointer after the work it enqueued has run, except kv_pool (kept for the
 * life of the cache).  HOST arrays are copied before the call returns.
 *
 * Errors.  A call returns a status right away for what the host can see (null
 * pointers, ids out of range, duplicate ids in one list, shapes the cache was
 * not created for); then nothing is enqueued.  What only the device can see
 * (a listed branch that is not active, pool exhaustion, a row buffer smaller
 * than the active list) makes the whole call a no-op on the device and stores
 * the status in a sticky device word; the first such status is kept until
 * sart_sync_status or sart_get_state returns and clears it.
 *
 * One cache may be used by one host thread at a time and on one stream at a
 * time (calls on different streams must be ordered by the caller).
 */
#ifndef SART_H
#define SART_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sart_cache sart_cache; /* opaque */

typedef enum {
  SART_OK = 0,
  SART_E_INVALID = 1,   /* bad argument, bad id, buffer too small              */
  SART_E_OOM_PAGES = 2, /* free stack holds fewer pages than the call needs    */
  SART_E_STATE = 3,     /* branch / request not in the state the call requires */
  SART_E_HIP = 4        /* a HIP runtime call failed; see sart_last_error      */
} sart_status;

/* Element type of the cache.  SART_FP8_E4M3 (an extension: the paper keeps KV in
 * the model's dtype, Section 5.1): Q, K, V cross the boundary as bf16; the pool
 * keeps K and V as 8-bit floats (OCP E4M3: 4 exponent bits, bias 7, 3 mantissa
 * bits, subnormals, largest finite 448): code = the E4M3 value nearest to the
 * exact quotient x / scale, ties to the even code, |x / scale| clamped to 448;
 * read back as value(code) * scale, with one float32 scale for K and one for V
 * per cache (k_scale, v_scale).  The library divides in float64, which decides
 * every code as the exact quotient does (a float32 division or a multiplication
 * by 1/scale would not).  Inputs must be finite.
 * Half the bytes of bf16 per cached token.  Needs page_tokens 16, head_dim 64 or
 * 128 and Hq/Hkv <= 16. */
typedef enum { SART_F32 = 0, SART_BF16 = 1, SART_FP8_E4M3 = 2 } sart_dtype;

#define SART_ALL_ACTIVE(rows) (-(rows))   /* n_seqs of sart_append_tokens: every active branch (count read on the
                                             device); k and v hold `rows` >= 1 rows */

typedef enum { SART_SEQ_PREFIX = 0, SART_SEQ_BRANCH = 1 } sart_seq_kind;

/* Branch life cycle (Algorithm 1: a branch leaves the batch by completing,
 * by the prune predicate, or by early stop). */
typedef enum {
  SART_BRANCH_UNUSED = 0,
  SART_BRANCH_ACTIVE = 1,
  SART_BRANCH_COMPLETED = 2,
  SART_BRANCH_PRUNED = 3,
  SART_BRANCH_EARLY_STOPPED = 4,
  SART_BRANCH_WAITING = 5       /* created, holds the prompt, not yet in the batch (see sart_start_branches) */
} sart_branch_state;

typedef enum {
  SART_PRUNE_DROP_LOWEST_K = 0, /* victims: the k lowest (score, handle) keys   */
  SART_PRUNE_KEEP_TOP_K = 1,    /* victims: all but the k highest keys          */
  SART_PRUNE_THRESHOLD = 2      /* Algorithm 1's predicate: score < threshold   */
} sart_prune_mode;

/* KV tile layouts inside a page (per KV head; K tile then V tile).
 *   NATURAL: K[token][d], V[token][d].
 *   MFMA16 : only bf16, page_tokens 16, head_dim 64 or 128, Hq/Hkv <= 16.
 *            16-byte chunks ordered so that one coalesced 1 KiB wave load is
 *            one matrix-core operand:
 *              K chunk (d/8)*16 + token          holds K[token][8*(d/8) .. +7]
 *              V chunk (d/32)*64 + (token/4)*16 + d%16
 *                      holds V[4*(token/4)+0..3][32*(d/32) + d%16]     then
 *                            V[4*(token/4)+0..3][32*(d/32) + 16 + d%16]
 *   MFMA16_FP8: the same for SART_FP8_E4M3, one byte per element, a 16-byte
 *            chunk holding what two bf16 chunks hold:
 *              K chunk (d/64)*64 + ((d/8)%4)*16 + token, byte 8*((d/32)%2) + d%8
 *              V chunk (d/64)*64 + (token/4)*16 + d%16,
 *                      byte 8*((d/32)%2) + 4*((d/16)%2) + token%4
 * The layout is chosen by sart_alloc_cache (MFMA16 whenever it applies unless
 * force_natural_layout is set) and reported by sart_cache_layout. */
typedef enum { SART_LAYOUT_NATURAL = 0, SART_LAYOUT_MFMA16 = 1, SART_LAYOUT_MFMA16_FP8 = 2 } sart_kv_layout;

typedef struct {
  int32_t n_layers;             /* >= 1: layers sharing the tables (see below)   */
  int32_t n_q_heads;            /* Hq                                            */
  int32_t n_kv_heads;           /* Hkv, divides Hq                               */
  int32_t head_dim;             /* d, multiple of 8, <= 256                      */
  int32_t page_tokens;          /* tokens per page (16 in every paper-like run)  */
  int32_t num_pages;            /* pages in the pool                             */
  int32_t max_requests;         /* request ids are 0 .. max_requests-1, used once*/
  int32_t branches_per_request; /* Nb                                            */
  int32_t finish_quota;         /* Q; 0 or > Nb disables early stop              */
  int32_t max_pages_per_branch; /* private pages a branch may hold               */
  int32_t max_prefix_pages;     /* pages a request's prompt may hold             */
  int32_t kv_dtype;             /* sart_dtype of Q, K, V (see sart_dtype)        */
  int32_t force_natural_layout; /* nonzero: never pick SART_LAYOUT_MFMA16        */
  void* kv_pool;                /* DEVICE, caller owned, or NULL: library owns   */
  size_t kv_pool_bytes;         /* >= sart_pool_bytes(desc) when kv_pool != NULL */
  const int32_t* initial_free_order; /* HOST [num_pages] permutation, or NULL =
                                        identity.  Page initial_free_order[0] is
                                        handed out first.                        */
  float k_scale;                /* SART_FP8_E4M3 only: scale of K, of V;         */
  float v_scale;                /* <= 0 means 1                                  */
  int32_t branches_start_waiting; /* nonzero: a request's Nb branches are created
                                   WAITING (Algorithm 1's queue of awaiting
                                   branches) and enter the batch one by one
                                   through sart_start_branches; 0: they are
                                   created ACTIVE, all at once                   */
} sart_cache_desc;

typedef struct {
  int32_t mode;                 /* sart_prune_mode                               */
  int32_t k;                    /* modes 0,1: per-request count                  */
  const int32_t* k_per_request; /* HOST [max_requests] or NULL (use k)           */
  const float* threshold;       /* HOST [max_requests], mode 2                   */
  const int32_t* max_pruned;    /* HOST [max_requests] or NULL (no cap): a request
                                   never exceeds this many pruned branches in
                                   total (Algorithm 1's max_num_pruned)          */
} sart_prune_policy;

/* Bytes of KV pool the description needs:
 * num_pages * page_tokens * 2 * Hkv * d * sizeof(element). */
size_t sart_pool_bytes(const sart_cache_desc* desc);

/* A0.  Creates the cache: every page free, no request, no branch (Sections 1 and
 * 2: the KV cache of the sampled branches is what limits how many can be batched,
 * so the pool, its free list and the branch tables are sized once, here).
 * Zero-fills the pool (so never-written slots hold finite values).  Synchronous.
 * On any error nothing stays allocated. */
sart_status sart_alloc_cache(const sart_cache_desc* desc, sart_cache** out);
sart_status sart_free_cache(sart_cache* cache);
int32_t sart_cache_layout(const sart_cache* cache); /* sart_kv_layout */

/* A1/A2.  Appends n_tokens[i] tokens of K and V to sequence ids[i], for i in
 * list order; rows of k and v are the sequences' tokens back to back,
 * DEVICE [sum n, Hkv, d] in kv_dtype.
 *   SART_SEQ_PREFIX: ids are request ids.  The first append to a request
 *     creates it together with its Nb active branches (Algorithm 1, Prefill:
 *     N branches pushed after prefilling), appended to the end of the active
 *     list in order j = 0..Nb-1, prefix reference count Nb.  Later prefix
 *     appends extend the prompt and are allowed until the first branch append
 *     of that request (SART_E_STATE after).  ids must not be NULL.
 *   SART_SEQ_BRANCH: ids are branch handles, all ACTIVE (else SART_E_STATE);
 *     ids == NULL means every active branch in active order and then n_seqs
 *     must equal the active count (else SART_E_INVALID), or be
 *     SART_ALL_ACTIVE(rows) = -rows: one token for every active branch, however
 *     many there are when the call executes (ids and n_tokens NULL; k and v
 *     hold `rows` rows, the library reads the first active-count of them; more
 *     active branches than rows: SART_E_INVALID, nothing changes).  That
 *     form stages no host data and bakes no count into the launch, so a decode
 *     step recorded into a HIP graph (this call, then sart_decode_attention
 *     with n_rows = capacity of q and out) can be replayed while branches are
 *     pruned or finished between replays.
 *   n_tokens == NULL means one token per sequence.
 * Layers.  All layers of a model share one set of tables (a token has the
 * same page and slot in every layer); the pool is [layer][page][kv head][K|V].
 * An append to layer 0 is the one that allocates pages and advances lengths.
 * An append to a layer > 0 writes that layer's K/V of the same tokens: it must
 * repeat the step's layer-0 append (same kind, list, counts; SART_E_INVALID at
 * once otherwise) and come before any other state-changing call; it changes no
 * state.  If that layer-0 append failed on the device, or a finish or prune
 * moved rows since, nothing is written and the status SART_E_STATE is stored
 * (sticky; after a failed layer-0 append its own status stays the first).
 * sart_decode_attention and sart_prefill_attention read the layer they name.
 * Pages are popped from the free stack sequence by sequence in list order,
 * each sequence taking its new pages in ascending logical page order.
 * Fewer free pages than needed: SART_E_OOM_PAGES, nothing changes. */
sart_status sart_append_tokens(sart_cache* cache, int32_t kind, int32_t n_seqs,
                               const int32_t* ids /*HOST*/,
                               const int32_t* n_tokens /*HOST*/,
                               const void* k /*DEVICE*/, const void* v /*DEVICE*/,
                               int32_t layer, void* stream);

/* A3-A6.  One decode step of attention (the batched decoding step of Algorithm 1,
 * Decode): for every active branch b (row a) and query head h,
 *   out[a,h,:] = sum_t softmax_t(scale * q[a,h,:] . K[t, h/G, :]) * V[t, h/G, :]
 * over t = the request's prompt tokens followed by b's own tokens (the token
 * appended this step included).  q: DEVICE [n_rows, Hq, d] kv_dtype;
 * out: DEVICE [n_rows, Hq, d] float; rows >= active count are left untouched.
 * n_rows < active count: SART_E_INVALID (sticky), nothing written.
 * scale <= 0 means 1/sqrt(d).  An empty context gives a zero row. */
sart_status sart_decode_attention(sart_cache* cache, int32_t layer,
                                  const void* q, float* out, int32_t n_rows,
                                  float scale, void* stream);

/* sart_decode_attention for callers that must not allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid device allocation.  Same
 * arguments, same result (bit for bit) and same errors as sart_decode_attention,
 * but the kernels' scratch (the partial results that the merge combines) is a
 * fixed array of SART_STATIC_SCRATCH_BYTES inside the library's device image
 * instead of memory the cache allocated: the call allocates and frees nothing.
 * Each GPU the library runs on holds that array until the process ends.
 * Limits: the cache's device must be current, and n_rows (counted up to
 * max_requests * Nb) must be small enough that the largest step it admits fits
 * the array,
 *   W + S + max(S, 4 W) <= (SART_STATIC_SCRATCH_BYTES - 256 KiB) / (4 * (G*d + pad4(2G)))
 * and S <= 65536, with W = 4 * workgroups of the decode launch (1024 by default)
 * and S = n_rows * Hkv; otherwise SART_E_INVALID and nothing is enqueued (configs
 * 2 and 4 of the paper-like workloads need 5632 and 7168 of 9126 and 12765).
 * All calls on one GPU share the array, whatever their cache or stream: calls
 * that overlap in time on one GPU race; the caller orders them. */
#define SART_STATIC_SCRATCH_BYTES (32u << 20)
sart_status sart_decode_attention_static(sart_cache* cache, int32_t layer,
                                         const void* q, float* out, int32_t n_rows,
                                         float scale, void* stream);

/* Prefill attention (Algorithm 1, Prefill; Section 4 takes the prefill phase
 * from plain LLM inference): causal self-attention over prompts already in the
 * cache.  For each listed request the queries are its LAST n_q[i] prompt tokens:
 * query j of the request sits at prompt position p = P - n_q[i] + j and reads
 * prompt tokens 0..p (itself included) through the request's prefix table;
 * out = softmax(q K^T * scale) V per query head, KV head = head / (Hq / Hkv).
 * n_q[i] = P: the whole prompt at once; smaller: one chunk of a chunked prefill
 * (append the chunk with sart_append_tokens(SART_SEQ_PREFIX), then attend with
 * the chunk's queries).  Decode branches of the request are not involved.
 *   request_ids, n_q   host arrays [n_seqs], n_seqs <= min(max_requests, 65535); ids in [0, max_requests), n_q >= 0;
 *   q                  device, [sum n_q][Hq][head_dim], kv_dtype, rows in list order;
 *   out                device, [sum n_q][Hq][head_dim], float32;
 *   scale              <= 0: 1 / sqrt(head_dim).
 * Errors: host-checkable faults return a status and enqueue nothing.  A request
 * that is not live (SART_E_STATE) or holds fewer than n_q[i] prompt tokens
 * (SART_E_INVALID) is found on the device: then nothing is written to out and
 * the status is sticky until sart_sync_status / sart_get_state reads it.
 * Asynchronous on `stream`; q and out are not retained after the stream work. */
sart_status sart_prefill_attention(sart_cache* cache, int32_t layer, int32_t n_seqs, const int32_t* request_ids,
                                   const int32_t* n_q, const void* q, float* out, float scale, void* stream);

/* A7.  Prunes branches by score (Algorithm 1, Decode: the pruning step).
 * scores: DEVICE float [n_scores], active order, n_scores >= active count.
 * Per request, over its active branches:
 *   DROP_LOWEST_K  the min(k, live) smallest keys (score, handle);
 *   KEEP_TOP_K     all but the min(k, live) largest keys;
 *   THRESHOLD      in ascending active index: score < threshold[r] and the
 *                  request's pruned count still below max_pruned[r].
 * In modes 0 and 1 max_pruned (if given) limits the victims to the lowest
 * keys that still fit under the cap.  A NaN score compares as +infinity.
 * Victims become PRUNED, their private pages return to the free stack at once,
 * the prefix is released when no branch of the request is left, and the
 * active list, lengths and block tables are compacted keeping order. */
sart_status sart_prune_branches(sart_cache* cache, const sart_prune_policy* policy,
                                const float* scores, int32_t n_scores, void* stream);

/* A8.  Marks the listed ACTIVE branches COMPLETED (Algorithm 1, Decode:
 * completed branches leave the batch), frees their pages, counts them, and when a
 * request has reached Q completions early-stops its remaining active branches
 * (Section 3, Solution 1).  Any listed branch not ACTIVE: SART_E_STATE,
 * nothing changes. */
sart_status sart_finish_branch(sart_cache* cache, int32_t n,
                               const int32_t* handles /*HOST*/, void* stream);

/* A waiting branch joins the batch (Algorithm 1, main scheduling workflow: while
 * the current batch has room, an awaiting branch is popped from the branch queue
 * and appended to it; Section 4: so the branches of a request need not start
 * decoding together).  Only for caches created with branches_start_waiting.
 * The listed branches, all WAITING (else SART_E_STATE, nothing changes), become
 * ACTIVE with no private tokens; each takes the place right after the last
 * active branch of its request, or, if the request has none, the end of the
 * active list (what inserting them one by one in list order gives), so a
 * request's branches stay neighbours in the active order; the rows behind them
 * move up with their block tables.  Until it starts a waiting branch holds its
 * request's prompt (it counts in prefix_refcnt) but no row of q, out or scores;
 * sart_prune_branches never sees it; when its request reaches Q completions it
 * is ended with the others (SART_BRANCH_EARLY_STOPPED). */
sart_status sart_start_branches(sart_cache* cache, int32_t n,
                                const int32_t* handles /*HOST*/, void* stream);

/* A branch splits (Section 2: tree search over reasoning trajectories expands
 * a trajectory into several continuations; the evaluation's Rebase baseline is
 * such a method).  Only for caches created with branches_start_waiting.
 * dst[i], a WAITING branch of the same request as src[i] (else SART_E_INVALID at
 * once), joins the batch as a copy of the ACTIVE branch src[i]: the same private
 * tokens so far, in every layer.  It takes its place like a started branch
 * (sart_start_branches: behind its request's last active branch; list order).
 * The two share the pages that are full at this moment - such a page is listed in
 * several rows of block_tables, at the same logical index, and returns to the
 * free stack when the last branch holding it ends, at that branch's turn of the
 * release order (Section 4's rule for the shared prompt, applied to what branches
 * have in common).  A partly filled last page is copied into a freshly popped
 * page (pops in list order), so every branch appends into a page of its own.
 * The same src may be listed several times; dst must not repeat.
 * Device-detected, sticky, nothing changes: a src that is not ACTIVE or a dst
 * that is not WAITING (SART_E_STATE); fewer free pages than partly filled pages
 * to copy (SART_E_OOM_PAGES).  sart_decode_attention reads shared pages once per
 * branch that holds them; only the prompt is read once per request. */
sart_status sart_fork_branches(sart_cache* cache, int32_t n, const int32_t* src /*HOST*/,
                               const int32_t* dst /*HOST*/, void* stream);

/* A8 without a host list: completes every active branch whose length (private
 * tokens) has reached target_len[handle] (DEVICE, max_requests * Nb entries, by
 * handle), exactly as sart_finish_branch would for the list of those branches
 * in active order (quota, early stop, release, compaction included).  No branch
 * qualifies: nothing changes.  Stages no host data, so a whole step - append
 * (SART_ALL_ACTIVE), attention, this call - can be recorded into a HIP graph
 * and replayed (Algorithm 1, Decode: completed branches leave the batch). */
sart_status sart_finish_reached(sart_cache* cache, const int32_t* target_len /*DEVICE*/, void* stream);

/* Waits for the cache's last-used stream, returns the sticky device status
 * and clears it. */
sart_status sart_sync_status(sart_cache* cache);

/* Waits, then copies the canonical integer state to HOST buffers (any may be
 * NULL).  Returns the sticky status like sart_sync_status.
 *   n_active        [1]
 *   active_handles  [max_requests*Nb]   first n_active valid, rest -1
 *   seq_lens        [max_requests*Nb]   private tokens, active order, rest 0
 *   block_tables    [max_requests*Nb, max_pages_per_branch]  active order, -1 padded (after sart_fork_branches
 *                   rows of one request may list the same page, at the same index)
 *   free_stack      [num_pages]         first free_top valid (top = last), rest -1
 *   free_top        [1]
 *   prefix_tables   [max_requests, max_prefix_pages]  -1 padded / released
 *   prefix_lens     [max_requests]      prompt tokens (kept after release)
 *   prefix_refcnt   [max_requests]      branches holding the prompt: active + waiting
 *   branch_state    [max_requests*Nb]   by handle
 *   req_counters    [max_requests, 2]   completed, pruned */
sart_status sart_get_state(sart_cache* cache, int32_t* n_active,
                           int32_t* active_handles, int32_t* seq_lens,
                           int32_t* block_tables, int32_t* free_stack,
                           int32_t* free_top, int32_t* prefix_tables,
                           int32_t* prefix_lens, int32_t* prefix_refcnt,
                           int32_t* branch_state, int32_t* req_counters);

/* DEVICE views of the active list for callers that keep their step loop on the
 * device (a recorded graph that gathers its per-branch inputs itself):
 * *active_handles -> int32[max_requests * Nb], the handles in active order
 * (entries past the active count are unspecified), *n_active -> one int32.
 * Owned by the library, read-only for the caller, valid until sart_free_cache;
 * their contents change with every state-changing call, in stream order. */
sart_status sart_device_views(sart_cache* cache, const int32_t** active_handles, const int32_t** n_active);

/* The decode step with rows addressed by branch handle, for a step loop that
 * never waits for the device (Algorithm 1, Decode: the batch decodes for T
 * steps between two maintenance rounds; the caller need not know which
 * branches are still in the batch to run them).  Row b of k, v, q and out
 * belongs to branch handle b, whatever its place in the active order; all four
 * hold max_requests * Nb rows; rows of branches that are not ACTIVE are neither
 * read nor written.  Otherwise sart_append_active_by_handle is
 * sart_append_tokens(SART_SEQ_BRANCH, SART_ALL_ACTIVE(max_requests * Nb), NULL,
 * NULL, k, v, layer) and sart_decode_attention_by_handle is
 * sart_decode_attention: same results for the same branches, same errors,
 * nothing staged from the host, so both replay from a HIP graph.  With
 * sart_finish_reached a whole step needs no gather by the caller and no state
 * read back. */
sart_status sart_append_active_by_handle(sart_cache* cache, const void* k, const void* v /*DEVICE [max_requests*Nb, Hkv, d]*/,
                                         int32_t layer, void* stream);
sart_status sart_decode_attention_by_handle(sart_cache* cache, int32_t layer, const void* q /*DEVICE [max_requests*Nb, Hq, d]*/,
                                            float* out /*DEVICE [max_requests*Nb, Hq, d]*/, float scale, void* stream);

/* The active count as of the last state-changing kernel that has run, read
 * without waiting for the device (the kernels store it to pinned host memory).
 * It lags the calls still queued: a loop that never reads the state back uses it
 * to notice, a few steps late, that the batch has drained.  -1: null cache. */
int32_t sart_active_count_hint(const sart_cache* cache);

/* Text of the last host-side error of this thread. */
const char* sart_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SART_H */
