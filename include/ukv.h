/*
 * ukv.h -- C ABI of the unified key-value cache decode path for MI355X (gfx950).
 *
 * The operations are the data-parallel steps behind the unified KV cache of SeaLLM
 * (arXiv 2504.15720, section 4.4 "Unified KV Cache" and the unified block manager of
 * section 5): several co-located LLM services share ONE pool of equal-sized blocks
 * ("pages", the paper's merged cache blocks); each request owns a block table that maps
 * its logical blocks to physical pages, and a second index locates data inside a page.
 *
 * Layout (all services, one attention layer per table).  A request's cache is a byte
 * stream: token-major, then kv-head-major, then K[head_dim] followed by V[head_dim] in
 * bf16.  One such K|V pair is a head-row of R = 4*head_dim bytes; a token occupies
 * T = n_kv_heads*R bytes (= n_kv_heads*head_dim*2*sizeof(bf16)).  Stream byte s lives in
 * physical page  page_table[table_off + s / page_bytes]  at in-page offset
 * s % page_bytes (the second index; it is derived, not stored).  page_bytes is a power of
 * two between 1 KiB and 1 MiB and must be a
 * multiple of every service's R, so a head-row never straddles pages; token rows may.
 * A request of n tokens owns ceil(n*T/page_bytes) pages.
 *
 * Conventions.
 *   - Every function returns UKV_OK (0) or a negative error code and never throws.
 *     ukv_last_error() gives a human-readable detail for the calling thread's last failure.
 *   - "HOST" pointers are read on the CPU during the call and may be reused on return.
 *     "DEVICE" pointers are HIP device memory owned by the caller and must stay valid
 *     until the work enqueued on `stream` has finished.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *     work and return without synchronising.  One pool must be driven from one stream at
 *     a time: calls on the same pool share staging and scratch buffers.
 *   - The compute calls do host work at call time (they plan the launch from the host arrays and write the
 *     per-call records into a staging slot), so a call recorded into a HIP graph would replay the batch it
 *     was recorded with; they are meant to be called, not captured.
 *   - The library never allocates or frees the pool memory itself.  It owns its host
 *     object, the free list and pinned, device-mapped staging buffers (per-call records); with
 *     UKV_PARAM_VALIDATE also one 256-byte device allocation per pool.
 *   - UKV_TRACE=1 in the environment: every compute call leaves one line on stderr when it returns,
 *     "ukv_trace call=<entry point> t_us=<host time since the first traced call> host_us=<time in the call>
 *     status=ok|error" followed by the call's work-list figures as key=value (requests, kv_bytes, sequences,
 *     items, spans, workgroups, ...).  Host time only; UKV_PARAM_PROFILE times the kernels.
 *   - What lives in host memory is checked during the call (service ids, lengths against the
 *     pool size, page ids of patches, alignment of offsets).  What lives in device memory is
 *     not: every page id the kernels find in page_table for a request's ceil(n*T/page_bytes)
 *     pages must be below the pool's page count (UKV_PARAM_VALIDATE turns on a check on the device),
 *     and the offset arrays must stay inside the caller's q / out / new_k / new_v / page_table
 *     allocations.
 *   - There is no CPU fallback: without a usable HIP device the compute calls fail with
 *     UKV_EHIP.
 */
#ifndef UKV_H
#define UKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define UKV_OK 0
#define UKV_EINVAL (-1) /* bad argument, unsupported shape, bad page id, double free */
#define UKV_ENOMEM (-2) /* free list exhausted (state unchanged) or host allocation failed */
#define UKV_ENOSPC (-3) /* caller-provided workspace or output array too small */
#define UKV_EHIP (-4)   /* a HIP runtime call failed */

#define UKV_MAX_SERVICES 16

typedef struct ukv_pool ukv_pool_t; /* opaque host object */

/* One co-located service, reduced to the shape of one attention layer.
 * Supported: head_dim 128 or 64 with n_q_heads = G * n_kv_heads, any G from 1 to 16
 * (the workloads' shapes -- G = 1, 4, 8 at head_dim 128, G = 1 at 64 -- are the ones the kernels are tuned for).
 * scale == 0 selects 1/sqrt(head_dim). */
typedef struct {
    uint32_t n_q_heads;
    uint32_t n_kv_heads;
    uint32_t head_dim;
    float scale;
} ukv_service_t;

/* base: DEVICE, page_bytes-aligned start of the pool; bytes: its size (a whole number of
 * pages is used).  page_bytes: power of two, >= 1024, multiple of every service's R. */
typedef struct {
    void *base;
    uint64_t bytes;
    uint32_t page_bytes;
    uint32_t n_services;
    const ukv_service_t *services; /* HOST [n_services] */
} ukv_pool_desc_t;

typedef struct {
    uint32_t n_q_heads, n_kv_heads, head_dim, group;
    uint32_t head_row_bytes; /* R */
    uint32_t token_bytes;    /* T */
    float scale;
    uint32_t heads_per_slice; /* kv heads one workgroup covers */
    uint32_t n_slices;        /* n_kv_heads / heads_per_slice */
    uint32_t token_lanes;     /* tokens a workgroup reads per iteration */
    uint64_t n_pages;
    uint64_t free_pages;
} ukv_service_info_t;

/* Unified block manager (section 5: the component that derives the block shape from the services' layer shapes
 * and hands out the pool's blocks): validates the services against the page size and builds a LIFO free list
 * that first hands out pages 0, 1, 2, ...  No device work. */
int ukv_pool_create(const ukv_pool_desc_t *desc, ukv_pool_t **out);
int ukv_pool_destroy(ukv_pool_t *pool);
int ukv_pool_info(const ukv_pool_t *pool, uint32_t service, ukv_service_info_t *out);

/* ceil(n_tokens * T / page_bytes) for the service; 0 on a bad argument. */
uint64_t ukv_pages_for_tokens(const ukv_pool_t *pool, uint32_t service, uint64_t n_tokens);

/* Pop n page ids (LIFO) into out_ids HOST [n].  UKV_ENOMEM leaves the free list unchanged. */
int ukv_pages_alloc(ukv_pool_t *pool, uint32_t n, int32_t *out_ids);
/* Push n page ids back, in order.  Out-of-range or already-free ids: UKV_EINVAL, list unchanged. */
int ukv_pages_free(ukv_pool_t *pool, uint32_t n, const int32_t *ids);

/* Mixed-service batch descriptor (structure of arrays).  Requests of different services may
 * be mixed freely; the paper's same-service batch (section 4.2) is the case of one service. */
typedef struct {
    uint32_t n_requests;
    const uint32_t *service_id; /* HOST [n] */
    const uint32_t *ctx_len;    /* HOST [n] tokens valid for attention (new token included) */
    const uint64_t *table_off;  /* HOST [n] entry offset of each request's table in page_table */
    int32_t *page_table;        /* DEVICE concatenated int32 page ids */
    const void *q;              /* DEVICE bf16, [n_q_heads][head_dim] per request */
    const uint64_t *q_off;      /* HOST [n] element offsets into q (multiples of 8) */
    void *out;                  /* DEVICE fp32, [n_q_heads][head_dim] per request */
    const uint64_t *out_off;    /* HOST [n] element offsets into out (multiples of 4) */
    const void *new_k;          /* DEVICE bf16 [n_kv_heads][head_dim] per request (append only) */
    const void *new_v;          /* DEVICE bf16, same layout (append only) */
    const uint64_t *new_off;    /* HOST [n] element offsets into new_k/new_v (multiples of 8) */
    uint32_t n_patches;         /* page-table entries to write before appending (may be 0) */
    const uint64_t *patch_entry; /* HOST [n_patches] entry index into page_table */
    const int32_t *patch_page;   /* HOST [n_patches] page id to store there */
} ukv_batch_t;

/* Store side of the cache (section 4.4: storing a step's KV pairs into merged blocks).
 * First writes the n_patches table entries, then copies request i's new K/V to token index
 * ctx_len[i]-1 of its stream, bit for bit.  Requests with ctx_len == 0 are skipped.  Uses
 * service_id, ctx_len, table_off, page_table, new_k, new_v, new_off and the patch arrays. */
int ukv_append(ukv_pool_t *pool, const ukv_batch_t *batch, void *stream);

/* Upper bound of the workspace ukv_decode_attention needs for ANY batch of at most
 * n_requests requests of this pool's services, under the current tunables. */
size_t ukv_decode_workspace_bytes(const ukv_pool_t *pool, uint32_t n_requests);

/* Decode phase (section 2.1: one new token per request attends to all cached KV pairs),
 * reading K/V through the block tables of the unified cache (section 4.4):
 *   out[i][a][:] = sum_t softmax_t(scale * q[i][a] . K[t][a/G]) * V[t][a/G],  t < ctx_len[i],
 * fp32 accumulation over bf16 inputs, fp32 output; ctx_len == 0 gives zeros.  Bytes of the
 * pool past ctx_len never influence the result (they may hold anything, NaN included); q and the K/V
 * of the tokens in [0, ctx_len) must hold finite values.  The batch is cut into token ranges that
 * run as one split-KV launch over all services; the workgroup that finishes a cut request
 * last merges its partial results (or a second launch does, see UKV_PARAM_FUSED_MERGE).
 * workspace: DEVICE, 256-byte aligned, ws_bytes >= ukv_decode_workspace_bytes(); else UKV_ENOSPC.
 * Uses service_id, ctx_len, table_off, page_table, q, q_off, out, out_off. */
int ukv_decode_attention(ukv_pool_t *pool, const ukv_batch_t *batch, void *workspace, size_t ws_bytes,
                         void *stream);

/* One decode iteration in one launch (section 2.1: each iteration stores the new token's KV pair and
 * attends over the whole cache; section 4.4: both go through the block table): the same results as
 * ukv_append followed by ukv_decode_attention on this batch -- pool bytes and page-table entries bit
 * for bit, out up to fp32 summation order.  The new page-table entries are written with the plan
 * upload; the workgroup that attends to a request's last token takes that token's K/V from
 * new_k/new_v, stores it into the request's pages and uses it from registers, so the store side
 * costs no launch of its own.  Arguments, workspace and errors as for those two calls together. */
int ukv_decode_step(ukv_pool_t *pool, const ukv_batch_t *batch, void *workspace, size_t ws_bytes, void *stream);

/* A decode plan that outlives its step.  ukv_decode_step plans every call on the host and uploads the plan; in
 * steady-state decoding the batch is the same from step to step and every request grows by one token, so the plan
 * made for one step serves the following ones: the growth goes to the last token range of every request, and the
 * only per-step data, the page ids of the table entries the growth needs, travel in the kernel arguments.  A step is
 * then ONE launch (plus the merge launch where UKV_PARAM_FUSED_MERGE is 0) with no host planning and no upload.
 * Results are those of ukv_decode_step on the same lengths: pool bytes and table entries bit for bit, out up to fp32
 * summation order.  The plan is remade (as in ukv_decode_step) on the first step, after UKV_PARAM_REPLAN_EVERY steps
 * (default 64: the cut drifts from balance as requests grow), after ukv_set_param, and for steps that do not fit the
 * kernel arguments (more than 766 requests or 576 new table entries).
 *   ukv_plan_create   batch: the requests as they are NOW (ctx_len tokens in the cache; patch fields ignored); the
 *                     host arrays are copied.  workspace: DEVICE, as for ukv_decode_step, owned by the plan until
 *                     ukv_plan_destroy; no device work.
 *   ukv_plan_step     advance != 0: every request grows by one token first.  Then, for every request, the token at
 *                     index ctx_len - 1 is stored from new_k / new_v (at the batch's new_off) and attention runs
 *                     over [0, ctx_len).  new_pages HOST [n_new_pages]: page ids for the table entries
 *                     ceil((c-1) T / P) .. ceil(c T / P) - 1 of each request (c its length in this step), in
 *                     request order; n_new_pages must be their exact number, else UKV_EINVAL and nothing changes.
 *                     io (may be NULL = the batch's pointers): other page table / q / out / new_k / new_v of the same
 *                     layout, e.g. the next layer of the same iteration, called with advance == 0 and that layer's
 *                     page ids.  While a plan is live the caller must not change the table entries of its requests.
 *   ukv_plan_lengths  the plan's current ctx_len, HOST [n] out. */
typedef struct ukv_plan ukv_plan_t;
typedef struct {
    int32_t *page_table; /* DEVICE */
    const void *q;       /* DEVICE bf16 */
    void *out;           /* DEVICE fp32 */
    const void *new_k;   /* DEVICE bf16 */
    const void *new_v;   /* DEVICE bf16 */
} ukv_plan_io_t;
int ukv_plan_create(ukv_pool_t *pool, const ukv_batch_t *batch, void *workspace, size_t ws_bytes, ukv_plan_t **out);
int ukv_plan_step(ukv_plan_t *plan, const ukv_plan_io_t *io, int advance, const int32_t *new_pages,
                  uint32_t n_new_pages, void *stream);
int ukv_plan_lengths(const ukv_plan_t *plan, uint32_t *ctx_len_out, uint32_t n);
int ukv_plan_destroy(ukv_plan_t *plan);

/* For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The same computation as ukv_decode_attention (results equal up to fp32 summation order), but
 *   - every array of the descriptor is DEVICE memory (nothing of the batch is read on the host, so the enqueued
 *     work follows whatever those arrays hold when it runs),
 *   - the launch is planned on the device, and the plan and the split-KV partials live in a device array of
 *     UKV_STATIC_SCRATCH_BYTES that is part of the library's code object: every GPU the library runs on holds one
 *     copy from the first use until the process ends,
 *   - the call allocates nothing (no device, pinned or staging memory, no events) and keeps no per-call state on
 *     the host; it enqueues four launches on `stream` (plan, decode, two merge kernels; no memset, no copy) and
 *     returns.  UKV_PARAM_PROFILE does not cover it.
 * Limits: n_requests <= UKV_STATIC_MAX_REQUESTS and n_requests * (largest n_slices of the pool's services, see
 * ukv_pool_info) <= 8192, else UKV_ENOSPC and nothing is enqueued; the device of the pool must be current.
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (different streams or
 * threads) race, and so would replays of two graphs that hold such calls; calls on one stream are safe.  The
 * array keeps the last call's contents; the plan kernel rewrites all of it that the next call reads.
 * What the host cannot check is the caller's duty, as for page ids: ctx_len[i] * T must fit the request's table
 * and the pool; a request whose service_id is not below the pool's service count is skipped (no output written). */
#define UKV_STATIC_SCRATCH_BYTES (16u << 20)
#define UKV_STATIC_MAX_REQUESTS 1024
typedef struct {
    uint32_t n_requests;
    const uint32_t *service_id; /* DEVICE [n] */
    const uint32_t *ctx_len;    /* DEVICE [n] */
    const uint64_t *table_off;  /* DEVICE [n] */
    const int32_t *page_table;  /* DEVICE */
    const void *q;              /* DEVICE bf16, as in ukv_batch_t */
    const uint64_t *q_off;      /* DEVICE [n] element offsets into q (multiples of 8) */
    void *out;                  /* DEVICE fp32 */
    const uint64_t *out_off;    /* DEVICE [n] element offsets into out (multiples of 4) */
} ukv_device_batch_t;
int ukv_decode_attention_static(ukv_pool_t *pool, const ukv_device_batch_t *batch, void *stream);

/* Prefill phase (section 2.1: the tokens of a prompt, or of a chunk of it, are processed in one pass
 * that leaves their KV pairs in the cache), attention part, causal:
 *   out[i][r][a][:] = sum_t softmax_t(scale * q[i][r][a] . K[t][a/G]) * V[t][a/G],  t <= ctx_len[i] - q_len[i] + r,
 * for the q_len[i] last tokens of request i (row r is the token at position ctx_len[i] - q_len[i] + r).
 * All ctx_len[i] tokens, the chunk's own included, must already be in the pool (ukv_scatter or
 * ukv_append) and hold finite values; bytes past ctx_len are never read.  q: DEVICE bf16 [q_len][n_q_heads][head_dim] per request at element offset q_off[i];
 * out: DEVICE fp32, same shape, at out_off[i]; q_len: HOST [n], 0 <= q_len[i] <= ctx_len[i].
 * fp32 accumulation as in ukv_decode_attention.  Every shape ukv_pool_create accepts is supported
 * (requests of head_dim 128 and of head_dim 64 run as two launches).  workspace: DEVICE, 256-byte aligned, at least
 * ukv_prefill_workspace_bytes(pool, n_requests, sum of q_len) bytes; else UKV_ENOSPC.
 * Uses service_id, ctx_len, table_off, page_table, q, q_off, out, out_off.
 *
 * The softmax weights reach the matrix cores in one of two forms (UKV_PARAM_PREFILL_WEIGHTS):
 *   two bf16 parts (16 significant bits; results within 3e-5 of exact arithmetic on unit-normal K, V and q), or
 *   one fp16 part (11 bits: every weight is off by at most 2^-11 of itself and the same rounded weights are summed
 *   for the denominator, so a result moves by at most 2^-10 times the largest distance of a V element of its row from
 *   it, and by that much only if every rounding error lined up with its V element; measured: within 5e-4 on
 *   unit-normal values -- and the kernel is 1.3 times faster).  The one-part form multiplies fp16 by
 *   fp16, so a first pass copies the V rows the call needs, as fp16, into the workspace (V elements beyond
 *   +-65504 saturate, elements below 2^-24 in magnitude become 0), which then has to hold
 *   ukv_prefill_workspace_bytes_one_part(pool, n_requests, sum of q_len, sum of ctx_len over the requests
 *   with q_len > 0) bytes.  By default the call takes the one-part form when the workspace is that large and the
 *   batch's attention (in flop) exceeds 35e9 plus 1500 per byte of that copy -- the cost of one more launch and of
 *   moving the copy, against a quarter of the kernel's time: whole prompts of a thousand tokens and more qualify,
 *   short chunks over long contexts do not -- and the two-part form otherwise.
 *
 * A workgroup takes 128 / G query rows of one (request, kv head) and walks the tokens they can see.  Where that gives few
 * workgroups with long walks (a chunk of a long prompt), the walks are cut into stretches of 1024 tokens or more, each a
 * workgroup that leaves a partial result in the workspace, merged by one more launch -- if the workspace has the room
 * that ukv_prefill_workspace_bytes_one_part includes for it (about 140 MB); else one workgroup per tile. */
size_t ukv_prefill_workspace_bytes(const ukv_pool_t *pool, uint32_t n_requests, uint64_t total_q_rows);
size_t ukv_prefill_workspace_bytes_one_part(const ukv_pool_t *pool, uint32_t n_requests, uint64_t total_q_rows,
                                            uint64_t total_ctx_tokens);
int ukv_prefill_attention(ukv_pool_t *pool, const ukv_batch_t *batch, const uint32_t *q_len, void *workspace,
                          size_t ws_bytes, void *stream);

/* Bulk load (also the tests' view of the pool): copy tokens [0, ctx_len[i]) of every request out of the pool into contiguous
 * k_out / v_out DEVICE bf16 [ctx_len][n_kv_heads][head_dim] at element offset kv_off[i] (HOST).
 * k_out / v_out (and k_in / v_in of the two calls below) may also be pinned host memory that the device
 * can address (hipHostMalloc): the kernel then moves the bytes over the host link itself, which is how
 * a preempted or migrating request's cache is swapped out and in (sections 4.2 and 5). */
int ukv_gather(ukv_pool_t *pool, const ukv_batch_t *batch, void *k_out, void *v_out, const uint64_t *kv_off,
               void *stream);

/* Bulk store: the inverse of ukv_gather.  Writes tokens [0, ctx_len[i]) of every request from
 * contiguous k_in / v_in DEVICE bf16 [ctx_len][n_kv_heads][head_dim] at element offset kv_off[i]
 * (HOST) into the request's pages, bit for bit.  This is how a prompt's K/V enter the cache after
 * the prefill phase (section 2.1), and, together with ukv_gather, how an ongoing request's cache
 * moves to another pool when the placement changes (request migration, section 5).  The table
 * entries for ceil(ctx_len*T/page_bytes) pages must already be in page_table. */
int ukv_scatter(ukv_pool_t *pool, const ukv_batch_t *batch, const void *k_in, const void *v_in,
                const uint64_t *kv_off, void *stream);

/* Bulk append: the store side of chunked prefill (section 2.1: the pass over a chunk of a prompt leaves the
 * chunk's KV pairs in the cache, behind those of the earlier chunks).  Writes the n_new[i] (HOST) LAST
 * tokens of request i, i.e. tokens [ctx_len[i] - n_new[i], ctx_len[i]), from contiguous k_in / v_in
 * DEVICE bf16 [n_new][n_kv_heads][head_dim] at element offset kv_off[i] (HOST, a multiple of 8), bit
 * for bit; tokens before the chunk are not touched.  n_new[i] = ctx_len[i] is ukv_scatter, n_new[i] = 1
 * the store of ukv_append, n_new[i] = 0 writes nothing.  UKV_EINVAL if n_new[i] > ctx_len[i].  The
 * table entries for ceil(ctx_len*T/page_bytes) pages must already be in page_table.
 * Uses service_id, ctx_len, table_off, page_table. */
int ukv_scatter_tokens(ukv_pool_t *pool, const ukv_batch_t *batch, const uint32_t *n_new, const void *k_in,
                       const void *v_in, const uint64_t *kv_off, void *stream);

/* Host-only view of the split-KV plan for a batch (no device work): how the launch would be cut. */
typedef struct {
    uint32_t n_seqs;        /* (request, head-slice) sequences */
    uint32_t n_items;       /* (sequence, token range) work items */
    uint32_t n_spans;       /* workgroups of the decode launch */
    uint32_t n_reduce;      /* sequences merged by the second launch */
    uint64_t partial_floats; /* fp32 values of split partials */
    uint64_t plan_bytes;     /* bytes copied to the device per call */
    uint64_t kv_bytes;       /* sum ctx_len * T: algorithmic KV bytes of the step */
} ukv_plan_info_t;
/* items_out (HOST, may be NULL): n_items_cap rows of {request, first kv head, n kv heads, t0, t1, span}. */
int ukv_plan_decode(const ukv_pool_t *pool, const ukv_batch_t *batch, ukv_plan_info_t *info,
                    uint32_t *items_out, uint32_t n_items_cap);

/* Tunables (integers).  Setting one never changes results beyond fp32 summation order. */
#define UKV_PARAM_MAX_SPANS 1        /* upper limit of decode workgroups per launch */
#define UKV_PARAM_MIN_SPAN_BYTES 2   /* do not cut spans smaller than this many KV bytes (default 512 KiB; until it is
                                        set, batches too small to fill the device that way are cut down to 64 KiB) */
#define UKV_PARAM_BLOCK_THREADS 3    /* 256 or 512 (default 512; 256 where every service has d = 128 and g > 1) */
#define UKV_PARAM_HEADS_PER_SLICE 4  /* 0 = automatic; else forced where it divides n_kv_heads */
#define UKV_PARAM_PROFILE 5          /* 0 = off; n >= 1 = time every n-th launch of each kernel with HIP events (see
                                        ukv_profile_read).  A timed launch costs about 10 us of stream time. */
#define UKV_PARAM_FUSED_MERGE 6      /* 1 = merge partials inside the decode launch; 0 = second launch (default: 1, and
                                        0 where every service has d = 128 and g > 1) */
#define UKV_PARAM_SLOTS 7            /* spans of the planner's first round; 0 (default) = one per compute unit of the device */
#define UKV_PARAM_GQA_COST_PCT 9     /* planner cost of a KV byte of a matrix-core service (d = 128, g > 1), in percent of
                                        a byte of the other kinds (default 150, measured on mixed batches) */
#define UKV_PARAM_PREFILL_XCD 10     /* 1 (default) = prefill workgroups of one (request, kv head) share an XCD (one L2) */
#define UKV_PARAM_REPLAN_EVERY 11    /* ukv_plan_step remakes its plan after this many tokens of growth (default 64; 0 = every step) */
#define UKV_PARAM_MERGE_ACQ_REL 12   /* merge inside the decode launch: 0 (default) = workgroups publish their partial results
                                        with agent-scope relaxed atomics, a wait for the store acknowledgements and a
                                        barrier before they count the item; 1 = the count is an agent-scope
                                        acquire-release, the ordering the language's memory model promises (4 to 8 % of
                                        the launch).  UKV_PARAM_FUSED_MERGE = 0 needs neither. */
#define UKV_PARAM_VALIDATE 13        /* 1 = before the kernels of a compute call run, a small kernel checks that every
                                        page-table entry the call will use names a page of the pool.  If one does not,
                                        the call's kernels do nothing (no read or write through the table), and the next
                                        compute call on the pool returns UKV_EINVAL, naming the entry (ukv_last_error).
                                        One extra launch per call (and 256 bytes of device memory per pool, allocated
                                        at the first checked call); default 0.  Not covered:
                                        ukv_decode_attention_static. */
#define UKV_PARAM_PREFILL_WEIGHTS 14 /* form of the softmax weights in ukv_prefill_attention: 0 (default) = one fp16 part
                                        where the workspace has room for the fp16 copy of V and the batch is large
                                        enough to pay for it, else two bf16 parts; 1 = always one part (UKV_ENOSPC if
                                        the workspace is too small); 2 = always two parts */
#define UKV_PARAM_PREFILL_FORM_USED 15 /* read only: the form the pool's last ukv_prefill_attention call took (1 or 2;
                                        0 before the first call) */
#define UKV_PARAM_PREFILL_PARTIALS_USED 16 /* read only: partial results the pool's last ukv_prefill_attention call made
                                        (0 = every tile of query rows was walked by one workgroup) */
#define UKV_PARAM_TAPER 8            /* 0 = equal spans; else spans shrink batch by batch, each batch of resident
                                        workgroups taking this percentage (5..95) of what is left; 1 = 88; default 1, and
                                        94 for pools whose services all have d = 128 and g > 1 */
int ukv_set_param(ukv_pool_t *pool, int key, int64_t value);
int ukv_get_param(const ukv_pool_t *pool, int key, int64_t *value);

/* Kernel times collected while UKV_PARAM_PROFILE is on (HIP events on the caller's stream).
 * Reading waits for the recorded events and resets the accumulators.  At most 8192 unread
 * timings are kept; past that the oldest are dropped. */
typedef struct {
    uint32_t n_decode, n_reduce, n_append, n_prefill;
    double decode_ms, reduce_ms, append_ms, prefill_ms; /* sums over the launches */
} ukv_profile_t;
int ukv_profile_read(ukv_pool_t *pool, ukv_profile_t *out);

const char *ukv_strerror(int code);
const char *ukv_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* UKV_H */
