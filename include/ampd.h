/*
 * ampd.h -- C ABI of libampd: batched incremental-prefill attention over a paged KV cache
 * for AMD MI355X (gfx950).
 *
 * The operation is the GPU work that a multi-round serving scheduler coordinates: a
 * prefill task with l_hist cached tokens and l_incr new tokens (initial prefill is the
 * l_hist = 0 case; paper Section 3, performance model T_pre(l_hist, l_incr)), a decode
 * step of one token per request (Section 3, T_dec; Section 1), an incremental prefill
 * executed locally on a decode instance next to its decode batch (Section 3, step 2,
 * "Local execution"), and the merge of incremental KV into the KV the decode worker
 * already stores (Section 3, step 2, "Remote execution", footnote).
 *
 * Notation: request r has C_r cached tokens and L_r new tokens, T_r = C_r + L_r.
 * Hq query heads, Hkv KV heads, G = Hq / Hkv, head dimension d, page size P.
 * New token i (0-based) of request r sits at absolute position C_r + i and attends keys
 * 0 .. C_r + i.  Query head hq reads KV head hq / G.
 *
 * Memory model
 *   - Every pointer is labelled HOST or DEVICE.  DEVICE pointers must belong to the GPU
 *     that is current on the calling thread.  The library never frees or retains caller
 *     pointers beyond the stream work it enqueues, and allocates no device memory.  Per
 *     device it keeps a ring of pinned host staging buffers for the work list (32 x 256 KiB,
 *     pinned by ampd_init or by the first attention call on that device) and one static
 *     device array of AMPD_STATIC_WORKSPACE_BYTES (see ampd_mixed_batch_attn_static).
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream) and the calls return without waiting for the GPU: a call takes a staging
 *     buffer that no enqueued copy still reads (the attention launch of a call marks its
 *     buffer free in a flag word the host polls), and when all are busy it pins one more, so the ring grows to the number of calls the caller keeps in
 *     flight (at 4096 buffers a call waits for the oldest instead).  The one exception is
 *     ampd_mixed_batch_attn_static, which may not allocate and waits for the oldest buffer.
 *   - HOST arrays are read before the call returns and may be reused immediately.
 *   - Threads: every entry point may be called from several host threads at once (the staging
 *     ring is shared under a lock; the last work list is kept per thread).  Calls that use the
 *     same workspace, output or pages must be ordered by the caller (same stream, or events).
 *
 * Layouts
 *   - Pools:  k_pool, v_pool  [num_pages][Hkv][P][d]  (row-major, bf16 bit patterns, or
 *     one byte per element for AMPD_KV_FP8_E4M3).  Token t of request r lives in page
 *     block_table[r][t / P], slot t % P.
 *   - Scales (8-bit cache only): k_scale, v_scale  float[num_pages][Hkv]; stored value =
 *     decode(code) * scale; scales are powers of two (see ampd_kv_append), and the attention
 *     kernels rely on it: they apply the exponent of a scale only.
 *   - Block table: int32 [num_reqs][max_pages_per_req], physical page ids.  Entries at
 *     index >= ceil(T_r / P) are never read (use -1).
 *   - Packed rows: q / out are bf16 [sum_r L_r][Hq][d], k_new / v_new bf16
 *     [sum_r L_r][Hkv][d]; the rows of request r start at the exclusive prefix sum of L.
 *   - Slots of the last page beyond T_r, unused pages and unused table entries are
 *     undefined memory: they never influence a result.
 *
 * Errors: every entry point validates its arguments on the host first.  On
 * AMPD_ERR_INVALID_ARG / UNSUPPORTED / WORKSPACE / PAGE_RANGE nothing has been enqueued.
 * AMPD_ERR_HIP reports a failed HIP call (launch, copy); work enqueued before it stays
 * enqueued.  Re-issuing a call with the same arguments is idempotent.
 */
#ifndef AMPD_H
#define AMPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    AMPD_OK = 0,
    AMPD_ERR_INVALID_ARG = -1,   /* NULL pointer, negative length, Hq % Hkv != 0, table too narrow */
    AMPD_ERR_UNSUPPORTED = -2,   /* head_dim not in {64,128}, page_size not in {16,32,64}, unknown kv_dtype */
    AMPD_ERR_WORKSPACE = -3,     /* workspace NULL, misaligned (256 B) or smaller than ampd_workspace_bytes() */
    AMPD_ERR_PAGE_RANGE = -4,    /* host mirror of the block table holds an id outside [0, num_pages) */
    AMPD_ERR_HIP = -5,           /* a HIP runtime call failed */
    AMPD_ERR_NOT_INITIALISED = -6 /* ampd_mixed_batch_attn_static before ampd_init on this device */
} ampd_status;

typedef enum { AMPD_KV_BF16 = 0, AMPD_KV_FP8_E4M3 = 1 } ampd_kv_dtype;

/* A persistent page pool.  All memory is owned by the caller. */
typedef struct {
    int32_t num_q_heads;      /* Hq  */
    int32_t num_kv_heads;     /* Hkv, divides Hq; Hq / Hkv <= 64 */
    int32_t head_dim;         /* d: 64 or 128 */
    int32_t page_size;        /* P: 16, 32 or 64 */
    int32_t kv_dtype;         /* ampd_kv_dtype */
    int32_t reserved;         /* must be 0 */
    int64_t num_pages;
    void *k_pool;             /* DEVICE [num_pages][Hkv][P][d] */
    void *v_pool;             /* DEVICE, same shape */
    float *k_scale;           /* DEVICE [num_pages][Hkv], NULL for bf16 */
    float *v_scale;           /* DEVICE [num_pages][Hkv], NULL for bf16 */
    float softmax_scale;      /* multiplies q.k before the softmax, e.g. 1/sqrt(d); finite, > 0 */
    int32_t reserved2;        /* must be 0 */
} ampd_kv_cache;

/* One batch: rows of (context length, incremental length).  L_r = 0 rows are no-ops,
 * C_r = 0 is an initial prefill, L_r = 1 is a decode row. */
typedef struct {
    int32_t num_reqs;
    int32_t max_pages_per_req;     /* row stride of the block table */
    const int32_t *h_ctx_len;      /* HOST [num_reqs], C_r >= 0 */
    const int32_t *h_incr_len;     /* HOST [num_reqs], L_r >= 0 */
    const int32_t *d_block_table;  /* DEVICE [num_reqs][max_pages_per_req] */
    const int32_t *h_block_table;  /* HOST mirror or NULL; when given, entries below ceil(T_r/P)
                                      are range-checked before anything is enqueued */
} ampd_batch;

/* Tuning knobs of the work planner; pass NULL for the defaults.  They change how the work
 * is cut, never the result beyond floating-point summation order. */
typedef struct {
    int32_t force_kv_splits;   /* > 0: cut every item's key range into exactly this many pieces
                                  (clamped to the number of 64-key tiles); 0 = automatic */
    int32_t reserved[7];       /* must be 0 */
} ampd_plan_options;

/* One-time set-up of the GPU that is current on the calling thread: pins the staging ring and
 * resolves the static workspace.  Optional for every call except ampd_mixed_batch_attn_static
 * (the others do the same set-up on their first use of a device); idempotent; thread-safe.
 * Returns AMPD_OK or AMPD_ERR_HIP. */
ampd_status ampd_init(void);

/* Bytes of DEVICE workspace the attention calls need for this batch (work list + split-KV
 * partial results), from the task metadata (l_hist, l_incr) alone (paper Section 3: the
 * scheduler holds these lengths on the CPU).  Pure host computation; returns 0 on invalid
 * arguments. */
size_t ampd_workspace_bytes(const ampd_kv_cache *cache, const ampd_batch *batch);
size_t ampd_workspace_bytes_opts(const ampd_kv_cache *cache, const ampd_batch *batch,
                                 const ampd_plan_options *opts);

/* Merge new K/V rows into the paged cache (paper Section 3, step 2, "Remote execution",
 * footnote: the decode worker merges the received incremental KV into the history KV it
 * stores; Section 3, step 4: it then holds all KV of the request): token i of request r is
 * written to position C_r + i.
 * k_new, v_new: DEVICE bf16 [sum L][Hkv][d].
 * bf16 cache: a bit-exact copy.  8-bit cache: per (page, KV head) and separately for K
 * and V, e = the smallest integer with amax <= 448 * 2^e over the tokens written to that
 * page by this call (clamped to [-40, 119]); if the page already held tokens of this
 * request (its first C_r mod P slots) the stored exponent is kept when it is >= e, else it
 * is raised to e and the old codes are re-encoded to the new scale; codes are E4M3
 * (OCP "fn": bias 7, max 448, no infinities) rounded to nearest, ties to even;
 * scale[page][head] = 2^e.  Inputs must be finite. */
ampd_status ampd_kv_append(const ampd_kv_cache *cache, const ampd_batch *batch,
                           const void *k_new, const void *v_new, void *stream);

/* The GPU side of a KV transfer between workers whose parallelism differs (paper Section 3,
 * T_kv(l_ctx; theta_src, theta_dst); Section 4.1, Eq. 2: history KV to the prefill worker,
 * incremental KV back): gather tokens [C_r, C_r + L_r) of every row, KV heads
 * [head_begin, head_begin + head_count) only, from the pages into packed rows
 * k_out, v_out: DEVICE bf16 [sum L][head_count][d] (the send buffer for the rank that owns those
 * heads), and the inverse scatter of received rows into pages.  bf16 caches only
 * (AMPD_ERR_UNSUPPORTED otherwise); bit-exact copies; h_ctx_len is the first token, h_incr_len
 * the token count of each row.  ampd_kv_unpack over all heads equals ampd_kv_append. */
ampd_status ampd_kv_pack(const ampd_kv_cache *cache, const ampd_batch *batch, int32_t head_begin,
                         int32_t head_count, void *k_out, void *v_out, void *stream);
ampd_status ampd_kv_unpack(const ampd_kv_cache *cache, const ampd_batch *batch, int32_t head_begin,
                           int32_t head_count, const void *k_in, const void *v_in, void *stream);

/* Append, then causal GQA attention of the L_r new queries of every row over its C_r + L_r
 * keys (paper Section 3, performance model T_pre(l_hist, l_incr): a prefill with history
 * l_hist = C_r and incremental length l_incr = L_r; initial prefill is l_hist = 0).
 * This and ampd_mixed_batch_attn are one implementation under two names: the planner turns
 * rows with few query rows into split-KV items and the others into prefill tiles, whatever
 * the entry point.
 * bf16 cache: the page writes ride in the attention launch as work items of their own and the
 * attention items read the new tokens from k_new / v_new (which, like every DEVICE argument,
 * must stay valid until the call's stream work is done).  8-bit cache: a quantising append
 * launch runs first and attention reads the quantised pages.
 * q: DEVICE bf16 [sum L][Hq][d];  out: DEVICE bf16 [sum L][Hq][d].
 * workspace: DEVICE, 256-byte aligned, >= ampd_workspace_bytes(). */
ampd_status ampd_incr_prefill_attn(const ampd_kv_cache *cache, const ampd_batch *batch,
                                   const void *q, const void *k_new, const void *v_new,
                                   void *out, void *workspace, size_t workspace_bytes,
                                   void *stream);

/* The same operation for a batch that mixes decode rows (L_r = 1; paper Section 3, T_dec:
 * one token per request per step) with incremental-prefill rows (L_r > 1) in any order, as
 * a decode instance executing prefills locally sees them (Section 3, step 2, "Local
 * execution"):
 * all attention work of the batch, compute-bound prefill tiles and bandwidth-bound decode
 * splits alike, is issued as ONE attention launch (followed by one combine launch when
 * key ranges were split). */
ampd_status ampd_mixed_batch_attn(const ampd_kv_cache *cache, const ampd_batch *batch,
                                  const void *q, const void *k_new, const void *v_new,
                                  void *out, void *workspace, size_t workspace_bytes,
                                  void *stream);

/* For callers that cannot allocate device memory (code that runs while a HIP graph is being
 * captured in the process, when hipMalloc is refused; tight serving loops; harnesses that
 * forbid allocation): ampd_mixed_batch_attn with the work list
 * and the split-KV partial results in a static device array of AMPD_STATIC_WORKSPACE_BYTES
 * that the library's code object carries (one copy per GPU, held until the process ends)
 * instead of a caller workspace.  The call allocates nothing, on the device or pinned:
 * ampd_init must have run on the current device (else AMPD_ERR_NOT_INITIALISED), and when all
 * staging buffers of the ring are still being read it waits for the oldest.  Batches whose
 * ampd_workspace_bytes() exceeds AMPD_STATIC_WORKSPACE_BYTES, or whose work list exceeds one
 * 256 KiB staging buffer (~5 000 work items), are rejected with AMPD_ERR_WORKSPACE before
 * anything is enqueued.  Results are bitwise those of ampd_mixed_batch_attn.  All calls on one
 * GPU share the array: calls on the same stream are ordered and safe, calls that overlap on
 * different streams of one GPU race.  Nothing in the array has to start at zero (every
 * partial result is written before it is read), so it is never cleared.  Like every
 * attention call it stages its work list on the host when it is made: recording the call
 * itself into a graph and replaying it is not supported. */
#define AMPD_STATIC_WORKSPACE_BYTES (32u << 20)
ampd_status ampd_mixed_batch_attn_static(const ampd_kv_cache *cache, const ampd_batch *batch,
                                         const void *q, const void *k_new, const void *v_new,
                                         void *out, void *stream);
size_t ampd_static_workspace_limit(void);   /* AMPD_STATIC_WORKSPACE_BYTES of the loaded library */

/* Variants taking planner options (NULL = defaults). */
ampd_status ampd_incr_prefill_attn_opts(const ampd_kv_cache *cache, const ampd_batch *batch,
                                        const void *q, const void *k_new, const void *v_new,
                                        void *out, void *workspace, size_t workspace_bytes,
                                        void *stream, const ampd_plan_options *opts);
ampd_status ampd_mixed_batch_attn_opts(const ampd_kv_cache *cache, const ampd_batch *batch,
                                       const void *q, const void *k_new, const void *v_new,
                                       void *out, void *workspace, size_t workspace_bytes,
                                       void *stream, const ampd_plan_options *opts);

/* Attention only (no append): the pools must already hold all C_r + L_r tokens (the state
 * after a remote execution's KV merge, paper Section 3, step 2).  Used to time the attention
 * launch alone and after a separate ampd_kv_append. */
ampd_status ampd_paged_attn(const ampd_kv_cache *cache, const ampd_batch *batch,
                            const void *q, void *out, void *workspace, size_t workspace_bytes,
                            void *stream, const ampd_plan_options *opts);

/* Description of the work list the planner builds for a batch from its (l_hist, l_incr)
 * metadata (host only; for tests and for the benchmark's roofline accounting).  Returns
 * AMPD_OK or a validation error. */
typedef struct {
    int64_t num_items;          /* attention work items (= workgroups of the attention launch), null items included */
    int64_t num_wide_items;     /* prefill tiles: up to 256 query rows, 8 waves share K/V tiles */
    int64_t num_narrow_items;   /* decode-style items: <= 32 query rows, 8 waves split the keys */
    int64_t num_combine_items;  /* query tiles whose key range was split */
    int64_t num_append_launches; /* append launches that precede the attention launch (8-bit cache; 0 for bf16) */
    int64_t partial_bytes;      /* split-KV partial results inside the workspace */
    int64_t plan_bytes;         /* work list inside the workspace */
    int64_t num_append_items;   /* bf16 cache: page-write items (64 packed rows each) that close the attention launch */
    int64_t num_workgroups;     /* workgroups of the attention launch: num_items, or 256 persistent workgroups that work
                                 * through the items when the launch holds tiles and more items than that */
} ampd_plan_info;
ampd_status ampd_plan_describe(const ampd_kv_cache *cache, const ampd_batch *batch,
                               const ampd_plan_options *opts, ampd_plan_info *info);

/* Copy the work items of an append-then-attend call, in launch order, to a HOST array of 10 int32 per item:
 * {request, kind (0 wide, 1 narrow, 2 null, 3 append), kv_head, first_head_in_group, heads, first_token, tokens,
 *  key_begin, key_end, partial_offset (-1: the item writes final output)};
 * an append item (bf16 cache) copies `tokens` consecutive packed rows of k_new / v_new, starting at new token
 * `first_token` of `request` and running on into the following requests, into their pages;
 * a null item (request -1) does no work: workgroup i runs on accelerator die i % 8, and null items keep
 * the wide items that follow on the die whose L2 holds their K/V stream;
 * writes at most max_items items, returns the total number (or a negative ampd_status). */
int64_t ampd_plan_items(const ampd_kv_cache *cache, const ampd_batch *batch,
                        const ampd_plan_options *opts, int32_t *h_items, int64_t max_items);

/* Last-resort timing hook: wall time in milliseconds of the most recent attention launch
 * and its combine launch on this thread, measured with HIP events recorded on the caller's
 * stream around them.  Only valid after the stream has been synchronised; returns
 * AMPD_ERR_INVALID_ARG if no launch was recorded or timing is disabled.
 * Timing is off by default; ampd_set_timing(1) turns it on for the CALLING THREAD only
 * (the flag and the events are per thread); this is the measurement hook behind the
 * offline profiling of T_pre / T_dec (paper Section 3, offline stage). */
void ampd_set_timing(int enabled);
ampd_status ampd_last_timing(float *attn_ms, float *combine_ms, float *append_ms);

const char *ampd_status_string(ampd_status s);
const char *ampd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AMPD_H */
