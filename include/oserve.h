/*
 * oserve.h - C ABI of the MI355X (gfx950) paged GQA decode-attention library.
 *
 * The operation: one decode step of attention for a batch of requests whose
 * context lengths differ widely (short compute-bound requests mixed with long
 * memory-bound ones: paper section 1 (i) and section 2, "Workload
 * heterogeneity").  Per section 2, "Phases of LLM inference", a decode step
 * takes the last generated token and the KV cache as inputs, so each query head
 * of each request holds ONE query vector that attends over all cached keys and
 * values of that request; the paper characterises this phase as
 * memory-bandwidth-bound (section 2; appendix C, "Decoding phase").  The cache
 * is held in fixed-size blocks (section 5.2, "KV cache transmission"); the
 * block ("page") size, the pool layout and the block-table format below are
 * this library's choices, the paper does not fix them.
 *
 * For request b, query head h, kv head j = h / (num_q_heads / num_kv_heads),
 * L = context_lens[b]:
 *
 *     k_t = k_pages[block_table[b][t / page_size]][j][t % page_size][:]   t = 0..L-1
 *     out[b][h][:] = sum_t softmax_t(scale * <q[b][h], k_t>) * v_t
 *
 * computed on the caller's stream by a split kernel (one wavefront per
 * (request, kv head, sequence split), online softmax, fp32 accumulation, bf16
 * MFMA) and a log-sum-exp merge of the splits; a third, tiny kernel first
 * expands the plan's records into one descriptor per work item in the workspace.
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its name ends in _host; `plan`
 *     objects are host objects owned by the library.
 *   - The caller owns all device memory, including `workspace`.  Launch calls
 *     never allocate or free device memory and never synchronise with the
 *     device, with one exception: a plan keeps OSERVE_PLAN_RING pinned staging
 *     slots for its records, so the (OSERVE_PLAN_RING+1)-th launch of a plan
 *     waits until the oldest launch's record copy has run on the device.
 *   - Every function returns a status code; nothing throws or aborts.
 *   - Objects are not synchronised: one plan (or migration) object must not be used by two
 *     threads at the same time; different objects are independent.
 *   - hipStream_t is passed as void* (null = the default stream).
 */
#ifndef OSERVE_H_
#define OSERVE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct oserve_plan oserve_plan_t;

typedef enum {
    OSERVE_OK = 0,
    OSERVE_ERR_NULL = 1,          /* a required pointer is null */
    OSERVE_ERR_SHAPE = 2,         /* unsupported head geometry, page size, batch or other size argument */
    OSERVE_ERR_CONTEXT_LEN = 3,   /* a context length < 1 or beyond the block-table width */
    OSERVE_ERR_WORKSPACE = 4,     /* workspace too small or misaligned */
    OSERVE_ERR_PLAN_MISMATCH = 5, /* batch larger than the plan's capacity, or plan has no device */
    OSERVE_ERR_DEVICE = 6,        /* a HIP runtime call failed */
    OSERVE_ERR_ALIGNMENT = 7      /* a device pointer is not aligned as the call requires */
} oserve_status_t;

/* Launches a plan may have in flight before a launch call waits for the oldest. */
#define OSERVE_PLAN_RING 8

/* Supported shapes: head_dim 64 or 128; page_size 16, 32 or 64; num_q_heads a
 * multiple of num_kv_heads with group size num_q_heads / num_kv_heads <= 16.
 * Split sizes are counted in tiles of 16 tokens (a page holds 1, 2 or 4 tiles), so
 * "pages" in the plan queries below means tiles; the two coincide at page_size 16. */

/*
 * Plan: sizes the sequence splits of one batch from its context lengths (the
 * step that lets short and long requests fill the GPU together).  With an
 * explicit `split_tokens` the sequence of request b (N_b pages) is cut into
 * S_b = ceil(N_b / C) splits of ceil(N_b / S_b) pages, C = split_tokens /
 * page_size.  With `split_tokens` = 0 the planner picks C (a multiple of 12
 * pages) as one resident wavefront's fair share of the batch (pages of the
 * batch x kv heads / wavefront slots of the device); requests of at most C
 * pages stay whole, and longer ones are cut into full-size splits followed by
 * a tail of splits that shrink (C, C/2, C/4, ... 12 pages) in proportion to
 * what is left of the request.  Work items (request, kv head, split) are
 * launched largest split first, so the small ones fill the end of the launch.
 * Host-only, O(batch log batch).
 *
 *   context_lens_host  [batch] int32, host memory, each in [1, max_pages_per_seq*page_size]
 *   max_pages_per_seq  row stride (entries) of the block table passed at launch
 *   split_tokens       0 = automatic; else a positive multiple of page_size
 *   device_id          HIP device on which the plan will be launched; its compute-unit and
 *                      SIMD counts (queried) size the splits; -1 = no device (planning
 *                      only, assumes 256 compute units of 4 SIMDs; such a plan cannot launch)
 *   capacity           largest batch a later oserve_plan_update may bring (>= batch)
 *
 * Errors: OSERVE_ERR_NULL, OSERVE_ERR_SHAPE, OSERVE_ERR_CONTEXT_LEN, OSERVE_ERR_DEVICE.
 * On error *plan_out is null.
 */
oserve_status_t oserve_plan_create(const int32_t* context_lens_host, int32_t batch,
                                   int32_t num_q_heads, int32_t num_kv_heads, int32_t head_dim,
                                   int32_t page_size, int32_t max_pages_per_seq,
                                   int32_t split_tokens, int32_t device_id, int32_t capacity,
                                   oserve_plan_t** plan_out);

/*
 * Re-plan in place for the next decode step (context lengths grow by one per
 * step, section 2 "step-by-step").  No allocation.  batch <= capacity.
 * On error the plan keeps its previous contents.
 */
oserve_status_t oserve_plan_update(oserve_plan_t* plan, const int32_t* context_lens_host,
                                   int32_t batch);

void oserve_plan_destroy(oserve_plan_t* plan); /* null is allowed; the plan's launches must have completed */

/* Plan queries (plan must be non-null). */
int32_t oserve_plan_batch(const oserve_plan_t* plan);
int32_t oserve_plan_num_work_items(const oserve_plan_t* plan); /* grid size of the split kernel */
int32_t oserve_plan_split_pages(const oserve_plan_t* plan);    /* C, in 16-token tiles */
int32_t oserve_plan_split_tokens(const oserve_plan_t* plan);   /* C, in tokens (16 x the above) */
/* Splits of request b: their count, and the size in 16-token tiles of its largest split.  Out pointers may be null. */
oserve_status_t oserve_plan_request(const oserve_plan_t* plan, int32_t b, int32_t* num_splits,
                                    int32_t* max_split_pages);
/* Inspection of the launch order: the plan holds oserve_plan_num_runs() runs, run i being `num_splits`
 * consecutive splits of `pages_per_split` pages of one request (the request's very last split may be
 * shorter), covering its logical pages [page_begin, page_end).  Runs are ordered largest split first;
 * run i owns work items [first_item, first_item + num_splits * num_kv_heads).
 * fields = {request, first_item, num_splits, pages_per_split, page_begin, page_end, row_base, total_splits}. */
int32_t oserve_plan_num_runs(const oserve_plan_t* plan);
oserve_status_t oserve_plan_run(const oserve_plan_t* plan, int32_t i, int32_t fields[8]);
/* Bytes of `workspace` the current plan needs, and a bound valid after any update. */
size_t oserve_plan_workspace_bytes(const oserve_plan_t* plan);
size_t oserve_plan_workspace_bytes_max(const oserve_plan_t* plan);

/*
 * One decode step of paged attention (definition at the top of this file).
 * Enqueues on `stream`: a one-workgroup kernel that reads the plan's records
 * from pinned host memory and writes the work-item descriptors into
 * `workspace`, the split kernel, and (if any request is split) the merge kernel.  Returns without waiting.  The records
 * are staged at call time, so the plan may be updated as soon as the call
 * returns; it must not be destroyed before the launch has run.
 *
 *   workspace      device, >= oserve_plan_workspace_bytes(plan), 256-byte aligned;
 *                  contents are scratch.  Two launches that overlap in time must
 *                  not share a workspace.
 *   q              bf16 [batch, num_q_heads, head_dim], contiguous
 *   k_pages        bf16 [num_pages, num_kv_heads, page_size, head_dim], contiguous (the tiles of a page follow
 *                  each other),
 *   v_pages        same shape; 16-byte aligned.  Slots at or beyond a request's context
 *                  length (in its last page) may be read but never influence the result,
 *                  whatever they hold; pages no table row names are never read.
 *   block_table    int32 [batch, max_pages_per_seq]: physical page of logical page p of
 *                  request b.  Only the first ceil(L_b / page_size) entries of a row are read.
 *   context_lens   int32 [batch], the device copy of the lengths the plan was built from.
 *                  The kernels take the split boundaries from the plan and from this array
 *                  only how many tokens of a request's last page count; a value that
 *                  disagrees with the plan is clamped into that page (no out-of-range read).
 *   scale          multiplies the fp32 score q.k (not q)
 *   out            fp32 [batch, num_q_heads, head_dim], contiguous
 *
 * Host-checked errors: OSERVE_ERR_NULL, OSERVE_ERR_WORKSPACE, OSERVE_ERR_PLAN_MISMATCH,
 * OSERVE_ERR_ALIGNMENT (q, k_pages, v_pages or out not 16-byte aligned), OSERVE_ERR_DEVICE.  Not checkable without a device round trip, hence undefined
 * behaviour: block-table entries outside the pool.
 */
oserve_status_t oserve_paged_decode_attn(oserve_plan_t* plan, void* workspace,
                                         size_t workspace_bytes, const void* q,
                                         const void* k_pages, const void* v_pages,
                                         const int32_t* block_table, const int32_t* context_lens,
                                         float scale, float* out, void* stream);

/*
 * The layers of a model.  A decode step runs every layer of the model on the same batch with
 * the same context lengths (section 2, "Phases of LLM inference": one token per step through
 * the whole model; section 5.2 speaks of the cache per layer), so the plan - and with it the
 * work-item descriptors that the first kernel of oserve_paged_decode_attn writes into the
 * workspace - is the same for all of them; only q, the K/V pools and out differ.
 * oserve_plan_stage enqueues that first kernel alone, once per step; each layer then calls
 * oserve_paged_decode_attn_staged, which enqueues only the split and merge kernels over the
 * descriptors already in `workspace` (the partial results in the workspace are reused layer
 * after layer, in stream order).  Results are bit-identical to oserve_paged_decode_attn.
 * The staged call enqueues kernels and nothing else (no copy, no event, no wait), so the
 * layers of a step may be captured into a HIP graph and replayed.  The calls that stage
 * records (oserve_plan_stage, oserve_paged_decode_attn, oserve_paged_decode_attn_static,
 * oserve_paged_mixed_attn, oserve_paged_prefill_attn) copy them into a pinned slot when they
 * are called and attach an event to their first kernel: call those eagerly, not under capture
 * (a replay would read whatever the slot holds by then).
 * The create and destroy calls allocate and free pinned memory and are not for capture either,
 * and the optional kernel timing (oserve_plan_enable_timing) must be off while capturing.
 *
 * The staged call checks on the host that `workspace` is the one the plan was last staged
 * into and that the plan has not been updated since (else OSERVE_ERR_PLAN_MISMATCH); all
 * these calls must go to one stream, or to streams the caller orders.  Other arguments and
 * errors: as oserve_paged_decode_attn.
 */
oserve_status_t oserve_plan_stage(oserve_plan_t* plan, void* workspace, size_t workspace_bytes, void* stream);
oserve_status_t oserve_paged_decode_attn_staged(oserve_plan_t* plan, void* workspace, size_t workspace_bytes,
                                                const void* q, const void* k_pages, const void* v_pages,
                                                const int32_t* block_table, const int32_t* context_lens,
                                                float scale, float* out, void* stream);

/*
 * The same decode step for callers that cannot allocate device memory: code that runs while a
 * HIP graph capture is in progress in the process (hipMalloc is not allowed then), tight
 * serving loops, harnesses that forbid hipMalloc.  Identical to
 * oserve_paged_decode_attn except that the workspace is a fixed array of
 * OSERVE_STATIC_WORKSPACE_BYTES bytes that the library holds in the memory of every GPU it is
 * loaded on, from load until the process ends.  The call itself allocates and frees nothing (no
 * hipMalloc, no hipFree, no allocating library routine) and enqueues the same three kernels.
 *
 *   - A plan whose oserve_plan_workspace_bytes() exceeds OSERVE_STATIC_WORKSPACE_BYTES is refused
 *     with OSERVE_ERR_WORKSPACE (the heterogeneous-mix benchmark batch needs 11 MB).
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU
 *     (different streams, or different threads) race, whatever plans they use.  Calls on one
 *     stream are ordered and safe.  The array keeps the previous call's contents; nothing in it
 *     has to be cleared between calls.
 *   - oserve_static_workspace_init(device) looks up the array's address on `device` ahead of
 *     time (set-up code; it may load the library's device code).  Without it the first
 *     oserve_paged_decode_attn_static call on a device does the look-up itself.
 * Other arguments, errors and undefined behaviour: as oserve_paged_decode_attn.
 */
#define OSERVE_STATIC_WORKSPACE_BYTES (32u << 20)
size_t oserve_static_workspace_bytes(void);
oserve_status_t oserve_static_workspace_init(int32_t device_id);
oserve_status_t oserve_paged_decode_attn_static(oserve_plan_t* plan, const void* q, const void* k_pages,
                                                const void* v_pages, const int32_t* block_table,
                                                const int32_t* context_lens, float scale, float* out,
                                                void* stream);

/*
 * Optional timing of the split kernel alone.  When enabled, each launch
 * attaches a begin and an end HIP event to the split kernel's dispatch on the
 * launch stream.
 * oserve_plan_split_kernel_ms waits for the launches recorded so far and
 * returns the mean split-kernel duration in milliseconds over all launches
 * since timing was enabled (enabling again resets the mean), and their count.
 */
oserve_status_t oserve_plan_enable_timing(oserve_plan_t* plan, int32_t enable);
oserve_status_t oserve_plan_split_kernel_ms(oserve_plan_t* plan, float* mean_ms, int32_t* count);

const char* oserve_status_string(oserve_status_t status);

/* ---------------------------------------------------------------------------
 * Chunked prefill over the same paged cache: the compute-bound side of the
 * batch (paper section 2, "Phases of LLM inference": the prefill phase
 * processes the prompt's tokens in parallel; section 1 (i): short requests are
 * compute-bound, long ones memory-bound).  Request b brings n_b = q_lens[b] new
 * query tokens whose keys and values already are the last n_b of its
 * L_b = context_lens[b] cached tokens.  Query token i (0 <= i < n_b) sits at
 * position p = L_b - n_b + i and attends causally:
 *
 *     out[r_b + i][h][:] = sum_{t <= p} softmax_{t <= p}(scale * <q[r_b + i][h], k_t>) * v_t
 *
 * with r_b = q_lens[0] + ... + q_lens[b-1] (the queries of all requests packed one
 * after the other), kv head and k_t, v_t as for the decode call.  n_b = 1 is a
 * decode step; a whole prompt is n_b = L_b.  A batch that holds decode requests
 * next to prefill chunks is served by oserve_paged_mixed_attn below.
 *
 * One workgroup of four wavefronts handles a block of 128 / G query tokens (G a power of two) of one
 * request against one kv head (G = num_q_heads / num_kv_heads), two workgroups per
 * compute unit; K and V tiles go through LDS; both products run on bf16 MFMA with
 * fp32 accumulation; the probabilities are rounded to bf16 for the second product and
 * normalised by the sum of the rounded values, so an output row is an exact convex
 * combination of value rows.
 * Supported shapes: head_dim 64 or 128; page_size 16, 32 or 64; G <= 16 (a group size that is not a
 * power of two is padded to the next one: the block then holds 128 / 2^ceil(log2 G) query tokens
 * and the padding columns are computed and dropped).
 * ------------------------------------------------------------------------- */
typedef struct oserve_prefill_plan oserve_prefill_plan_t;

/*
 * Plan: the list of work items (block of query tokens x kv head).  The blocks of one
 * (request, kv head) read the same K/V; they are placed at launch indices that are
 * equal modulo the device's XCD count (queried; 8 without a device) so that they run
 * side by side on one XCD and share its L2; (request, kv head) groups are dealt to the XCDs heaviest first.
 * Host-only.  It also owns the pinned staging through which the kernel reads that
 * list (OSERVE_PLAN_RING slots, same reuse rule as the decode plan).
 *
 *   context_lens_host  [batch] int32 host, L_b in [1, max_pages_per_seq * page_size]
 *   q_lens_host        [batch] int32 host, n_b in [1, L_b]
 *   device_id          HIP device the plan will be launched on; -1 = planning only
 *   capacity           largest batch a later update may bring (>= batch)
 *   max_query_tokens   largest sum of n_b a later update may bring
 *
 * Errors: OSERVE_ERR_NULL, OSERVE_ERR_SHAPE, OSERVE_ERR_CONTEXT_LEN (a length out of
 * range or n_b > L_b), OSERVE_ERR_PLAN_MISMATCH (more query tokens than max_query_tokens),
 * OSERVE_ERR_DEVICE.  On error *plan_out is null.
 */
oserve_status_t oserve_prefill_plan_create(const int32_t* context_lens_host, const int32_t* q_lens_host,
                                           int32_t batch, int32_t num_q_heads, int32_t num_kv_heads,
                                           int32_t head_dim, int32_t page_size, int32_t max_pages_per_seq,
                                           int32_t device_id, int32_t capacity, int64_t max_query_tokens,
                                           oserve_prefill_plan_t** plan_out);
/* Re-plan in place; no allocation.  On error the plan keeps its previous contents. */
oserve_status_t oserve_prefill_plan_update(oserve_prefill_plan_t* plan, const int32_t* context_lens_host,
                                           const int32_t* q_lens_host, int32_t batch);
void oserve_prefill_plan_destroy(oserve_prefill_plan_t* plan); /* null allowed; launches must have completed */
int32_t oserve_prefill_plan_num_work_items(const oserve_prefill_plan_t* plan);
int64_t oserve_prefill_plan_query_tokens(const oserve_prefill_plan_t* plan);  /* sum of n_b */
int32_t oserve_prefill_plan_block_tokens(const oserve_prefill_plan_t* plan);  /* query tokens per work item */
/* Item i of the launch order: fields = {request, kv_head, q_begin, q_row0, context_len, q_len}. */
oserve_status_t oserve_prefill_plan_item(const oserve_prefill_plan_t* plan, int32_t i, int32_t fields[6]);

/*
 * Enqueues the prefill kernel on `stream` and returns without waiting (except for
 * the staging-slot reuse described above).  All pointers are device pointers:
 *   q            bf16 [sum n_b, num_q_heads, head_dim], contiguous, 16-byte aligned
 *   k_pages,
 *   v_pages      as for oserve_paged_decode_attn; slots at or beyond L_b may hold anything
 *   block_table  int32 [batch, max_pages_per_seq]
 *   scale        multiplies the fp32 score; must be positive and finite
 *   out          fp32 [sum n_b, num_q_heads, head_dim], contiguous
 * Host-checked errors: OSERVE_ERR_NULL, OSERVE_ERR_SHAPE (scale), OSERVE_ERR_ALIGNMENT, OSERVE_ERR_PLAN_MISMATCH
 * (plan without device), OSERVE_ERR_DEVICE.  Block-table entries outside the pool: undefined.
 */
oserve_status_t oserve_paged_prefill_attn(oserve_prefill_plan_t* plan, const void* q, const void* k_pages,
                                          const void* v_pages, const int32_t* block_table, float scale,
                                          float* out, void* stream);
/* Optional timing of the kernel, as oserve_plan_enable_timing / oserve_plan_split_kernel_ms. */
oserve_status_t oserve_prefill_plan_enable_timing(oserve_prefill_plan_t* plan, int32_t enable);
oserve_status_t oserve_prefill_plan_kernel_ms(oserve_prefill_plan_t* plan, float* mean_ms, int32_t* count);


/* ---------------------------------------------------------------------------
 * Mixed batches: decode requests and prefill chunks in one call (paper section 1 (i)
 * and section 2, "Workload heterogeneity": the requests of one batch differ widely, short
 * ones compute-bound and long ones memory-bound; section 2, "Phases of LLM inference":
 * the compute-intensive prefill phase and the memory-bandwidth-bound decoding phase).
 * Same definition as oserve_paged_prefill_attn: request b brings n_b = q_lens[b] query
 * tokens, the rows of q and out are packed request after request, and query token i of
 * request b attends causally to the cached tokens 0 .. L_b - n_b + i.  What differs is
 * how the work is run: requests with n_b = 1 are decode requests and go through the
 * split-sequence decode work items (HBM-bound, then the log-sum-exp merge), requests with
 * n_b > 1 through the prefill work items (MFMA-bound), and ONE kernel holds both kinds at
 * the same time on every compute unit: the launch has two workgroups of four wavefronts
 * (one per SIMD) per compute unit, which last for the whole launch; the four wavefronts of
 * the one work through a queue of prefill items together, those of the other each through
 * a queue of decode items, so that every SIMD runs a prefill wavefront's MFMAs next to a
 * decode wavefront's K/V stream.  When one queue runs dry its workgroups turn to the other.
 * Supported shapes: as oserve_paged_prefill_attn (head_dim 64 or 128; G <= 16).
 * ------------------------------------------------------------------------- */
typedef struct oserve_mixed_plan oserve_mixed_plan_t;

/*
 * Plan (host-only): the decode work items of the requests with n_b = 1 (sized as by
 * oserve_plan_create with split_tokens = 0, queued largest first) and the prefill work items
 * of the others (blocks of 128 / G query tokens x kv heads, one queue per XCD so that the blocks
 * of one (request, kv head) share an L2).  Arguments and errors as oserve_prefill_plan_create.
 */
oserve_status_t oserve_mixed_plan_create(const int32_t* context_lens_host, const int32_t* q_lens_host,
                                         int32_t batch, int32_t num_q_heads, int32_t num_kv_heads,
                                         int32_t head_dim, int32_t page_size, int32_t max_pages_per_seq,
                                         int32_t device_id, int32_t capacity, int64_t max_query_tokens,
                                         oserve_mixed_plan_t** plan_out);
/* Re-plan in place; no allocation.  On error the plan keeps its previous contents. */
oserve_status_t oserve_mixed_plan_update(oserve_mixed_plan_t* plan, const int32_t* context_lens_host,
                                         const int32_t* q_lens_host, int32_t batch);
void oserve_mixed_plan_destroy(oserve_mixed_plan_t* plan); /* null allowed; launches must have completed */
int64_t oserve_mixed_plan_query_tokens(const oserve_mixed_plan_t* plan);   /* sum of n_b: rows of q and out */
/* counts = {workgroups of the mixed kernel (= 2 x compute units), prefill work items, decode work items,
 * prefill queues (= XCDs)}. */
oserve_status_t oserve_mixed_plan_counts(const oserve_mixed_plan_t* plan, int32_t counts[4]);
/* Prefill item i (queue after queue, each in the order it is worked through):
 * fields = {queue, request, kv_head, q_begin, q_row0, context_len, q_len}. */
oserve_status_t oserve_mixed_plan_prefill_item(const oserve_mixed_plan_t* plan, int32_t i, int32_t fields[7]);
size_t oserve_mixed_plan_workspace_bytes(const oserve_mixed_plan_t* plan);
size_t oserve_mixed_plan_workspace_bytes_max(const oserve_mixed_plan_t* plan);

/*
 * Enqueues on `stream`: the kernel that copies the plan's records from pinned host memory into
 * `workspace` and clears the queue counters, the mixed kernel, and (if a decode request is split)
 * the merge kernel.  Returns
 * without waiting, allocates nothing (same staging-ring rule as oserve_paged_decode_attn).
 *   workspace      device, >= oserve_mixed_plan_workspace_bytes(plan), 256-byte aligned, scratch
 *   q              bf16 [sum n_b, num_q_heads, head_dim], contiguous, 16-byte aligned
 *   k_pages, v_pages, block_table   as for oserve_paged_decode_attn
 *   context_lens   int32 [batch], device copy of the lengths the plan was built from (read for the
 *                  decode requests only, as in oserve_paged_decode_attn)
 *   scale          multiplies the fp32 score; must be positive and finite
 *   out            fp32 [sum n_b, num_q_heads, head_dim], contiguous
 * Host-checked errors: OSERVE_ERR_NULL, OSERVE_ERR_SHAPE (scale), OSERVE_ERR_WORKSPACE,
 * OSERVE_ERR_ALIGNMENT, OSERVE_ERR_PLAN_MISMATCH, OSERVE_ERR_DEVICE.
 */
oserve_status_t oserve_paged_mixed_attn(oserve_mixed_plan_t* plan, void* workspace, size_t workspace_bytes,
                                        const void* q, const void* k_pages, const void* v_pages,
                                        const int32_t* block_table, const int32_t* context_lens, float scale,
                                        float* out, void* stream);
/* Optional timing of the mixed kernel, as oserve_plan_enable_timing / oserve_plan_split_kernel_ms. */
oserve_status_t oserve_mixed_plan_enable_timing(oserve_mixed_plan_t* plan, int32_t enable);
oserve_status_t oserve_mixed_plan_kernel_ms(oserve_mixed_plan_t* plan, float* mean_ms, int32_t* count);


/* ---------------------------------------------------------------------------
 * KV-block migration copies (paper section 5.2, "KV cache transmission": at a
 * deployment switch the KV blocks of long requests are migrated in batched,
 * layer-aligned chunks into buffers pre-allocated on the target, which may hold
 * a different share of the kv heads).  One layer's chunk, on one GPU:
 *
 *   gather : stage[s][j][:][:] = pool[table[row_r][s - first_r]][head_begin + j][:][:]
 *   scatter: pool[target_table[r][s - first_r]][head_begin + j][:][:] = stage[s][j][:][:]
 *
 * for every migrating request r (in the order given at creation), staging page
 * s in [first_r, first_r + ceil(L_r / page_size)) and copied head j in
 * [0, num_heads).  Pools are bf16 [pages, pool_kv_heads, page_size, head_dim],
 * staging chunks bf16 [num_pages, num_heads, page_size, head_dim], both for K
 * and for V.  Pure data movement: results are bit-exact.
 * ------------------------------------------------------------------------- */
typedef struct oserve_kv_migration oserve_kv_migration_t;

/*
 * The migrating requests.  Host-only except for one device array of 16 bytes per
 * staging page (which table entry names the page), allocated here and owned by
 * the object (this call synchronises).
 *   context_lens_host  [num_requests] int32 host: L_r >= 1
 *   table_rows_host    [num_requests] int32 host: row of request r in the SOURCE block table
 *   device_id          -1 = host object only (cannot launch)
 * Errors: OSERVE_ERR_NULL, OSERVE_ERR_SHAPE, OSERVE_ERR_CONTEXT_LEN, OSERVE_ERR_DEVICE.
 */
oserve_status_t oserve_kv_migration_create(const int32_t* context_lens_host, const int32_t* table_rows_host,
                                           int32_t num_requests, int32_t page_size, int32_t device_id,
                                           oserve_kv_migration_t** out);
void oserve_kv_migration_destroy(oserve_kv_migration_t* m);   /* null allowed; launches must have completed */
int64_t oserve_kv_migration_num_pages(const oserve_kv_migration_t* m);   /* pages of a staging chunk */
/* First staging page and page count of request r.  Out pointers may be null. */
oserve_status_t oserve_kv_migration_request(const oserve_kv_migration_t* m, int32_t r, int32_t* first_page,
                                            int32_t* num_pages);
/*
 * Enqueue one copy on `stream` (no allocation, no synchronisation).  Device pointers, 16-byte aligned.
 * gather reads rows table_rows_host[r] of `block_table`; scatter reads row r of `target_block_table`.
 * max_pages_per_seq is the row stride of the table and must cover the longest migrating request.
 * Pages the tables do not name, and heads outside [head_begin, head_begin + num_heads), are not touched.
 * Host-checked errors: OSERVE_ERR_NULL, OSERVE_ERR_SHAPE, OSERVE_ERR_ALIGNMENT, OSERVE_ERR_PLAN_MISMATCH,
 * OSERVE_ERR_DEVICE.  Table entries outside the pool, or two requests naming one target page: undefined.
 */
oserve_status_t oserve_kv_gather(oserve_kv_migration_t* m, const void* k_pool, const void* v_pool,
                                 const int32_t* block_table, int32_t max_pages_per_seq, int32_t pool_kv_heads,
                                 int32_t head_begin, int32_t num_heads, int32_t head_dim, void* k_stage,
                                 void* v_stage, void* stream);
oserve_status_t oserve_kv_scatter(oserve_kv_migration_t* m, const void* k_stage, const void* v_stage,
                                  const int32_t* target_block_table, int32_t max_pages_per_seq,
                                  int32_t pool_kv_heads, int32_t head_begin, int32_t num_heads, int32_t head_dim,
                                  void* k_pool, void* v_pool, void* stream);
/* Optional timing of the copy kernel (latest launch folded into a running mean), as for the other kernels. */
oserve_status_t oserve_kv_migration_enable_timing(oserve_kv_migration_t* m, int32_t enable);
oserve_status_t oserve_kv_migration_kernel_ms(oserve_kv_migration_t* m, float* mean_ms, int32_t* count);


/* ---------------------------------------------------------------------------
 * Host-side planners of the serving method (no GPU work; every pointer is a
 * HOST pointer).
 * ------------------------------------------------------------------------- */

/*
 * Greedy switch plan (paper section 5.2 and the appendix "Greedy Algorithm for Ad
 * Hoc Model Switching"): for every model shard m and every target device t that
 * needs m and does not hold it, choose the source device that sends it.  Sources
 * on t's machine are preferred to sources on other machines; among the candidates
 * the one with the least volume already planned from it to t is chosen (the first
 * listed among equals), and the pair's counter grows by the shard's volume.
 * Shards are processed in index order, targets in the order listed.
 *
 *   device_machine   [num_devices] machine index of each device
 *   source_offsets   [num_shards + 1], source_devices: the devices holding shard m are
 *                    source_devices[source_offsets[m] .. source_offsets[m+1])
 *   target_offsets   [num_shards + 1], target_devices, volumes: likewise the devices that
 *                    need shard m and the volume of each such (m, t) requirement
 *   chosen_source    out, aligned with target_devices: the chosen source, or -1 where the
 *                    target already holds the shard
 *   pair_load        out or null: [num_devices x num_devices] planned volume from s (row) to t
 * Errors: OSERVE_ERR_NULL, OSERVE_ERR_SHAPE (bad index, negative volume, a needed shard nobody holds).
 */
oserve_status_t oserve_switch_plan(int32_t num_devices, const int32_t* device_machine, int32_t num_shards,
                                   const int32_t* source_offsets, const int32_t* source_devices,
                                   const int32_t* target_offsets, const int32_t* target_devices,
                                   const int64_t* volumes, int32_t* chosen_source, int64_t* pair_load);

/*
 * Edge capacity normalisation (section 4.2): the common capacity M of a replica that
 * can process per_type_capacity[j] requests of type j per unit time alone is the least
 * common multiple of those numbers (zeros = types it cannot serve are skipped); one
 * type-j request then consumes units_per_request[j] = M / per_type_capacity[j] units.
 * Errors: OSERVE_ERR_NULL, OSERVE_ERR_SHAPE (negative capacity, overflow of 64 bits).
 */
oserve_status_t oserve_capacity_normalise(const int64_t* per_type_capacity, int32_t num_types, int64_t* common,
                                          int64_t* units_per_request);

/*
 * Lower-level workload assignment (section 4.2): the assignment x[k][j] >= 0 of type-j
 * requests to replica k that serves the most requests subject to
 *   C1  sum_k x[k][j] <= arrivals[j]
 *   C2  x[k][j] <= edge_capacity[k][j]                 (skipped when edge_capacity is null or infinite)
 *   C3  sum_j x[k][j] * M_k / node_capacity[k][j] <= M_k   (M_k as in oserve_capacity_normalise)
 * Because the types consume different shares of a replica per request, this flow
 * problem is a linear program; it is solved exactly (simplex).  The optimum value
 * `total` is unique; the assignment attaining it need not be.
 *   arrivals       [num_types]
 *   node_capacity  [num_replicas x num_types] int64, 0 = replica cannot serve the type
 *   edge_capacity  [num_replicas x num_types] or null
 *   assignment     out [num_replicas x num_types], total: out
 * Errors: OSERVE_ERR_NULL, OSERVE_ERR_SHAPE (negative or non-finite input, more than 4096 pairs).
 */
oserve_status_t oserve_assign_workload(int32_t num_replicas, int32_t num_types, const double* arrivals,
                                       const int64_t* node_capacity, const double* edge_capacity,
                                       double* assignment, double* total);

#ifdef __cplusplus
}
#endif
#endif /* OSERVE_H_ */
