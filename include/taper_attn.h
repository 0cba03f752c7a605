/*
 * taper_attn -- decode-step attention over a paged bf16 KV cache whose parallel
 * branches share their request's prefix pages (MI355X / gfx950).
 *
 * One decode step is one forward pass that advances every admitted sequence by
 * one token (paper §1, §2.3).  A sequence is a serial request or one admitted
 * branch of a request in a parallel phase.  By the visibility rule (paper §3.1)
 * a branch token attends to the request's shared prefix followed by the branch's
 * own private tokens and to nothing of its siblings; the shared prefix is stored
 * once and served to all branches "from a single set of prefix blocks" (§3.1),
 * a branch materialising only its branch-local tokens (App. C, memory
 * accounting).  The time this call takes is the attention term of the step
 * latency T(S) that the admission controller budgets against (§3.2, App. C).
 *
 * All entry points are plain C.  "host" / "device" after a pointer says where the
 * memory must live.  Every function returns 0 on success or a negative
 * taper_status; none throws or aborts.  taper_last_error() gives a message for
 * the calling thread's last failure.
 *
 * ---------------------------------------------------------------- data layout
 * q, out : bf16 [n_seqs][n_q_heads][head_dim], row-major, device.
 * lse    : f32  [n_seqs][n_q_heads], device (optional): natural-log normaliser
 *          log sum_t exp(scale * q.k_t).
 * kv_pages (the pool), device: bf16 [n_pool_pages][2][n_kv_heads][page_size*head_dim];
 *          index 0 of the second axis is K, 1 is V.  Inside one
 *          (page, K, kv head) tile, element (tok, d) is at
 *                (d / 8) * (page_size * 8) + tok * 8 + d % 8
 *          i.e. K is stored in groups of 8 dims: [head_dim/8][page_size][8].
 *          Inside one (page, V, kv head) tile, element (tok, d) is at
 *                (tok / 4) * (4 * head_dim) + d * 4 + tok % 4
 *          i.e. V is stored transposed in groups of 4 tokens: [page_size/4][head_dim][4].
 *          Both are what a 64-lane MFMA operand fetch reads with unit stride.
 *          Slots past a segment's length and unreferenced pages may hold any
 *          bit pattern, NaN and Inf included; results do not depend on them.
 * Grouped-query attention: query head h reads KV head h / (n_q_heads / n_kv_heads).
 *
 * ---------------------------------------------------------------- the batch
 * block_table[s][*] (int32, host, row stride bt_row_stride): the physical pages
 *   of sequence s in logical order: first ceil(prefix_len[s]/page_size) entries
 *   are the request's shared prefix pages (identical for all members of a
 *   request), then ceil(suffix_len[s]/page_size) private pages.  Private tokens
 *   start on a fresh page even if the prefix ends mid-page.
 * branch_group[s] (int32, host): request id; starts at 0, non-decreasing in steps
 *   of 1, members of one request contiguous.
 * prefix_len[s], suffix_len[s] (int32, host): shared and private token counts
 *   (P ++ H and h_i ++ y_{i,<t} of §3.1).  prefix_len is equal inside a request.
 *   A serial request is a group of one; its context may be given as prefix,
 *   suffix or both.  prefix_len + suffix_len >= 1.
 */
#ifndef TAPER_ATTN_H
#define TAPER_ATTN_H

#include <stdint.h>

#if defined(__GNUC__)
#define TAPER_API __attribute__((visibility("default")))
#else
#define TAPER_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TAPER_OK = 0,
    TAPER_EINVAL = -1, /* null pointer, unsupported shape, bad argument            */
    TAPER_EBLOCK = -2, /* block-table entry < 0 or >= n_pool_pages                 */
    TAPER_EGROUP = -3, /* group ids not contiguous / prefix differs inside a group */
    TAPER_ELEN = -4,   /* negative length, empty context, row too short            */
    TAPER_EHIP = -5,   /* HIP runtime error, or a device call on a host-only ctx   */
    TAPER_ENOMEM = -6  /* host or device allocation failed                         */
} taper_status;

/*
 * How the partial result of one work item travels to the workgroup that merges a
 * sequence's partials (a sequence whose context is cut into several work items;
 * one that is a single item never goes through a partial).  Accumulation is fp32
 * in registers either way, and so are the running max and sum of every partial.
 */
typedef enum {
    TAPER_PARTIAL_F16_SCALED = 0, /* default: the accumulator row, divided by its own sum (a weighted mean
                                     of V rows) and by a power of two that brings its largest magnitude
                                     into [0.5, 1), in half precision; the power of two travels in fp32
                                     beside the running max and sum.  Error 2^-12 of the row's largest
                                     element, whatever the magnitude of V (no range limit); half the
                                     workspace traffic of fp32 rows                                        */
    TAPER_PARTIAL_F32 = 1         /* the accumulator row divided by its own sum, in fp32                   */
} taper_partial_format;

typedef struct {
    int n_q_heads;  /* 64 (Qwen3-32B shape, App. D) or any multiple of n_kv_heads  */
    int n_kv_heads; /* 8                                                            */
    int head_dim;   /* 64 or 128                                                    */
    int page_size;  /* 16                                                           */
    float scale;    /* softmax scale, normally 1/sqrt(head_dim)                     */
    int device;     /* HIP device ordinal; -1 = host-only context: plans can be
                       built, validated and exported, device calls return TAPER_EHIP */
    int partial_format; /* taper_partial_format; 0 = default                        */
} taper_attn_config;

typedef struct taper_ctx taper_ctx;   /* owns the partials workspaces             */
typedef struct taper_plan taper_plan; /* owns host + device copies of the step's integer metadata */

/* One unit of KV streaming: n_tokens tokens starting at block-table entry page0 of
 * row seq0, multiplied against the query rows of n_branch consecutive sequences. */
typedef struct {
    int32_t seq0;      /* first sequence; its block-table row supplies the pages    */
    int32_t n_branch;  /* sequences seq0..seq0+n_branch-1 share these tokens        */
    int32_t page0;     /* first block-table entry of the chunk                      */
    int32_t n_tokens;  /* valid tokens in the chunk (>= 1)                          */
    int32_t part_base; /* first partial row; row of (kv head hk, branch b, head-in-group j)
                          = part_base + hk * n_branch * gqa + b * gqa + j           */
    int32_t kind;      /* 0 = shared prefix of a parallel request, 1 = private, 2 = private
                          and the sequence's only item (result written directly, no partial),
                          3 = like 2 and run by a single wave (runs of short sequences)      */
    int32_t part;      /* workgroup share this item belongs to; n_parts for pool items */
    int32_t merge0;    /* merge_start[seq0]: where the merge entries of the item's sequences begin */
} taper_work_item;

/* Where sequence s finds one of its partials: rows first_row + hk*rows_per_head + j */
typedef struct {
    int32_t first_row;
    int32_t rows_per_head;
} taper_merge_entry;

/* Read-only view of a plan's host-side integers (valid until taper_plan_free). */
typedef struct {
    int32_t n_seqs, n_groups;
    const int32_t *ctx_len;        /* [n_seqs] prefix_len + suffix_len                      */
    const int32_t *n_prefix_pages; /* [n_seqs] ceil(prefix_len / page_size)                 */
    const int32_t *n_suffix_pages; /* [n_seqs] ceil(suffix_len / page_size): the branch's
                                      marginal blocks (App. C), 0 for an empty branch       */
    const int32_t *group_start;    /* [n_groups + 1] CSR of requests over sequences         */
    const int32_t *seg_start;      /* [n_seqs + 1] CSR of private segments over sequences   */
    const int32_t *seg_len;        /* tokens of each private segment                        */
    const int32_t *seg_page0;      /* block-table entry each private segment starts at      */
    int32_t n_items;
    const taper_work_item *items;  /* [n_items], ordered by part, then the n_pool_items pool items */
    int32_t n_pool_items;
    int32_t n_parts_shared, n_parts_private;
    const int32_t *part_start;     /* [n_parts_shared + n_parts_private + 1] CSR over items */
    const int32_t *merge_start;    /* [n_seqs + 1] CSR over merge entries                   */
    const taper_merge_entry *merge;
    int64_t n_partial_rows;
    int64_t tokens_unique;  /* sum over requests of prefix_len + sum over sequences of suffix_len */
    int64_t tokens_logical; /* sum over sequences of prefix_len + suffix_len: L_context of §3.2   */
    int32_t workspace_id;   /* which of the context's workspaces the plan is bound to (counts from 1 in
                               order of creation); it never changes while the plan lives          */
    int64_t workspace_rows; /* partial rows that workspace holds                                  */
} taper_plan_view;

typedef struct {
    int32_t target_workgroups; /* workgroups the KV stream is cut for; 0 = default: two per compute unit
                                  of the context's device (512 on MI355X, and on a host-only context) */
    int32_t share_prefix;      /* 1 = default: read each request's prefix once for all its
                                  branches; 0 = every branch streams the prefix by itself  */
    int32_t max_branches_per_item; /* 0 = default (head_dim 128: 12 row tiles, 24 branches at 8
                                      query heads per KV head; head_dim 64: 8 row tiles); wider
                                      requests are cut into equal sub-groups of at most this
                                      size; at most 12 row tiles                               */
    int32_t shared_cost_pct;   /* 0 = default (160 when no shared item is wider than 4 row tiles,
                                  200 up to 8, 140 above at head_dim 128): cost of a
                                  shared-prefix token relative to a private one when cutting
                                  the work into equal shares                                    */
    int32_t shared_item_cost;  /* 0 = default (800): fixed cost of a shared-prefix item, in private
                                  tokens' streaming time                                       */
    int32_t private_item_cost; /* 0 = default (128): fixed cost of a private item, same unit      */
    int32_t private_merge_cost; /* 0 = default (192 when the step has shared-prefix work, else none),
                                  -1 = none: extra cost of the private item that ends a sequence
                                  (as a rule it delivers the last partial and merges)           */
    int32_t solo_item_tokens;  /* 0 = default (512), -1 = never: sequences that are one item of at most this
                                  many tokens are run by single waves, four side by side, where a share
                                  holds at least 4 of them in a row                               */
    int32_t min_share_tokens;  /* a small step is cut into fewer shares than target_workgroups allows
                                  rather than into shares below this size.  0 = default: 256, or 1/16
                                  of the longest private segment if that is more (keeps the partials
                                  of one sequence to about 16)                                   */
    int32_t pool_pct;          /* 0 = default (25 when the step has shared-prefix work, else none):
                                  percentage of the private tokens that no share owns; workgroups
                                  that finish their share take them, an item at a time, so the
                                  launch ends evenly.  -1 = none; values above 90 count as 90    */
    int32_t pool_item_tokens;  /* size of the pool's items, rounded down to a multiple of 32 tokens (at
                                  least 32); 0 = default: a quarter of a share, between 512 and 1536 */
    int32_t small_step_grid;   /* 0 = default: when target_workgroups is 0, a step without shared-prefix work
                                  is cut for one workgroup per compute unit instead of two if that cuts
                                  sequences into so many fewer pieces that it pays (each piece costs
                                  partial rows and a share of a merge); 1 = the same rule for an explicit
                                  target_workgroups (then halved); -1 = never                    */
    int32_t scatter_sub_groups; /* 0 = default: the sub-groups of a request wider than
                                  max_branches_per_item get the same cuts, a share per item and
                                  neighbouring workgroups, so that they stream the prefix in step
                                  and share it in the L2; 1 = they are placed like unrelated
                                  requests, one after the other                               */
} taper_plan_options;

TAPER_API int taper_create(const taper_attn_config *cfg /* host */, taper_ctx **out_ctx);
TAPER_API void taper_destroy(taper_ctx *ctx);

/*
 * Workspaces.  The partial rows and arrival counters of a launch live in a
 * workspace owned by the context.  A plan is bound, when it is built, to the
 * context's current workspace if that is large enough; otherwise a larger one is
 * allocated BESIDE it and becomes current.  A workspace is never freed or moved
 * while a plan bound to it lives, so launches already enqueued, and HIP graphs
 * captured from a plan, stay valid for as long as their plan does, whatever is
 * built afterwards.  Superseded workspaces no plan is bound to any more are
 * released at the next growth (after a device synchronisation) and in
 * taper_destroy; in the steady state nothing is allocated, freed or synchronised.
 *
 * taper_reserve sizes the current workspace ahead of time for plans of up to
 * max_seqs sequences and max_partial_rows partial rows (n_partial_rows of a
 * representative plan's view; a host-only context computes it without a GPU), so
 * that no later taper_plan_build allocates.  TAPER_EINVAL for negative sizes,
 * TAPER_ENOMEM when the device allocation fails.  On a host-only context only
 * the bookkeeping is done.
 *
 * The arrival and pool counters of a workspace are zero between launches (every
 * launch leaves them so).  They are cleared when a workspace is created, and
 * again, on the stream of the next taper_plan_build or launch, after any call on
 * the context has reported a HIP error.
 */
TAPER_API int taper_reserve(taper_ctx *ctx, int max_seqs, int64_t max_partial_rows);

/*
 * Index resolution for one decode step (paper: the engine's batch formation
 * precedes the forward pass, App. D "Serving engine"; which pages each query row
 * reads follows §3.1).  Validates the batch, derives the request CSR, page counts,
 * the list of KV chunks and the merge map, copies them to the device on
 * `hip_stream` (unless the context is host-only) and binds the plan to a
 * workspace (see taper_reserve: a larger one is allocated beside the current one
 * if the plan needs it).  The host arrays are only read during the call.  One plan
 * serves every layer of the step.  Not safe to call concurrently on one ctx.
 * Plans must be freed before their context is destroyed; a freed plan's buffers
 * are recycled by later plans of the same context, ordered on the stream.
 * opts may be NULL.
 */
TAPER_API int taper_plan_build(taper_ctx *ctx, int n_seqs, const int32_t *block_table /* host */, int bt_row_stride,
                     const int32_t *branch_group /* host */, const int32_t *prefix_len /* host */,
                     const int32_t *suffix_len /* host */, int64_t n_pool_pages,
                     const taper_plan_options *opts /* host, may be NULL */, void *hip_stream,
                     taper_plan **out_plan);
/*
 * The same with a LIST of private segments per sequence (reduce-phase visibility,
 * paper §3.1: a reduce token attends to the shared prefix, then to every
 * completed branch in canonical order, then to the reduce tokens so far).
 * Sequence s sees prefix_len[s] prefix tokens and then the segments
 * seg_len[seg_start[s] .. seg_start[s+1]) in that order.  Its block-table row
 * lists the prefix pages and then each segment's pages; every segment starts on
 * a fresh page (so the pages a branch wrote during the parallel phase are
 * listed as they are, partially filled last page included) and an empty
 * segment owns no page.  taper_plan_build is the case of one segment per
 * sequence.  In the plan's view suffix_len-derived fields are totals over a
 * sequence's segments.  TAPER_EINVAL for a malformed CSR.
 */
TAPER_API int taper_plan_build_segments(taper_ctx *ctx, int n_seqs, const int32_t *block_table /* host */,
                                        int bt_row_stride, const int32_t *branch_group /* host */,
                                        const int32_t *prefix_len /* host */, const int32_t *seg_start /* host */,
                                        const int32_t *seg_len /* host */, int64_t n_pool_pages,
                                        const taper_plan_options *opts /* host, may be NULL */, void *hip_stream,
                                        taper_plan **out_plan);
TAPER_API void taper_plan_free(taper_plan *plan);
TAPER_API int taper_plan_export(const taper_plan *plan, taper_plan_view *out_view /* host */);

/*
 * Physical slot id (page * page_size + token-in-page) of every logical position:
 * slots[s * stride + t] for t < ctx_len[s], -1 after.  The host form reads the
 * plan's host copy; the device form runs a kernel over the very device arrays the
 * attention kernels index with, and writes `slots` in device memory.
 */
TAPER_API int taper_plan_resolve_slots_host(const taper_plan *plan, int64_t *slots /* host */, int64_t stride);
TAPER_API int taper_plan_resolve_slots(taper_ctx *ctx, const taper_plan *plan, int64_t *slots /* device */, int64_t stride,
                             void *hip_stream);

/*
 * The hot call (paper §1/§2.3 decode step; §3.1 visibility rule): for every
 * sequence s and query head h,
 *     out[s,h,:] = sum_t softmax_t(scale * q[s,h,:].K_t) V_t
 * over t in shared prefix ++ private tokens of s.  Enqueues one kernel on
 * `hip_stream` and returns; allocates nothing, does not synchronise.  q, kv_pages,
 * out (and lse if not NULL) are device pointers owned by the caller and must stay
 * valid until the stream has run the work.  Partial results of a sequence that is
 * cut into several work items travel in the context's taper_partial_format.
 * Calls on one ctx share its workspaces and must be ordered on one stream.  The
 * call may be recorded into a HIP graph (stream capture) and replayed while the
 * plan lives (the graph holds the addresses of the plan's device arrays and of the
 * workspace the plan is bound to, both of which live as long as the plan): the
 * kernel leaves its counters at zero and nothing else is enqueued.
 */
TAPER_API int taper_decode_step_attention(taper_ctx *ctx, const taper_plan *plan, const void *q /* device */,
                                const void *kv_pages /* device */, void *out /* device */,
                                float *lse /* device, may be NULL */, void *hip_stream);

/* Same operation with the batch arrays passed directly: builds a transient plan,
 * runs the step and frees the plan after synchronising the stream. */
TAPER_API int taper_decode_step_attention_simple(taper_ctx *ctx, int n_seqs, const void *q /* device */,
                                       const void *kv_pages /* device */, int64_t n_pool_pages,
                                       const int32_t *block_table /* host */, int bt_row_stride,
                                       const int32_t *branch_group /* host */, const int32_t *prefix_len /* host */,
                                       const int32_t *suffix_len /* host */, void *out /* device */,
                                       void *hip_stream);

/*
 * For callers that cannot allocate device memory -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: the operation and arguments of
 * taper_decode_step_attention_simple, but the plan's device arrays and the partials
 * workspace (counters, statistics, partial rows) live in a fixed 64 MiB array that is part
 * of the library's device image, one copy per GPU, held until the process ends.  The call
 * allocates and frees nothing, on the device or in pinned memory (its pinned staging buffer
 * and the array's address are set up by taper_create), and unlike _simple it only enqueues
 * (an upload of the plan, a clear of the counters, the decode kernel) and returns; the host
 * arrays are read during the call only.  No lse output.
 * TAPER_EINVAL with a message naming the sizes when the step needs more than the array holds
 * (plan image above 8 MiB, or image + workspace above 64 MiB: the 64-layer admission-sweep batch at
 * 640 sequences takes 30 MiB), TAPER_EHIP on a host-only context or when the array's address
 * could not be looked up.
 * All calls on one GPU, from any context, share that GPU's array, which keeps the previous
 * call's contents: a call must not be enqueued before every earlier one on that GPU has been
 * ordered before it (same stream, or an event); calls that overlap on one GPU race.
 */
TAPER_API int taper_decode_step_attention_static(taper_ctx *ctx, int n_seqs, const void *q /* device */,
                                       const void *kv_pages /* device */, int64_t n_pool_pages,
                                       const int32_t *block_table /* host */, int bt_row_stride,
                                       const int32_t *branch_group /* host */, const int32_t *prefix_len /* host */,
                                       const int32_t *suffix_len /* host */, void *out /* device */,
                                       void *hip_stream);

/*
 * Step-latency probe (paper App. C "Fitting": wall-clock latency of synthetic
 * steps; §2.3: externality E = T(S(k)) - T(S0)).  Runs `warmup` untimed and
 * `iters` timed steps; a step enqueues the attention of n_layers layers (layer l
 * uses q[l], kv[l], out[l]) with one plan.  Each step is bracketed by HIP events
 * on `hip_stream`.  The call synchronises the stream.
 */
typedef struct {
    double us_min, us_median, us_mean; /* per step (all layers)                       */
    int32_t n_tokens;                  /* sequences in the step (n_tokens of App. C)  */
    int32_t n_layers;
    int64_t l_context;                 /* aggregate context length (L_context)        */
    int64_t kv_bytes_unique;           /* per layer, prefix counted once per request  */
    int64_t kv_bytes_logical;          /* per layer, prefix counted once per sequence */
    double gbps_unique, gbps_logical;  /* from us_median                              */
} taper_probe_result;

TAPER_API int taper_step_latency_probe(taper_ctx *ctx, const taper_plan *plan, int n_layers,
                             const void *const *q_per_layer /* host array of device ptrs */,
                             const void *const *kv_per_layer /* host array of device ptrs */,
                             void *const *out_per_layer /* host array of device ptrs */, int warmup, int iters,
                             void *hip_stream, taper_probe_result *result /* host */);

/*
 * Duration of the decode kernel (the one launch a layer's attention consists of:
 * shared-prefix work, private work and the merge of partials) measured with HIP
 * events on `hip_stream` (synchronises).  us[0] = mean, us[1] = minimum over
 * `iters` launches after `warmup`.
 */
TAPER_API int taper_kernel_times(taper_ctx *ctx, const taper_plan *plan, const void *q, const void *kv_pages, void *out,
                       int warmup, int iters, void *hip_stream, double us[2] /* host */);
/* The same with launch i running on layer i mod n_layers (its q, pool and out): with enough
 * distinct pools no launch finds KV of an earlier one in the 256 MB Infinity Cache, which
 * repeated launches over one small pool do. */
TAPER_API int taper_kernel_times_layers(taper_ctx *ctx, const taper_plan *plan, int n_layers,
                              const void *const *q_per_layer /* host array of device ptrs */,
                              const void *const *kv_per_layer /* host array of device ptrs */,
                              void *const *out_per_layer /* host array of device ptrs */, int warmup, int iters,
                              void *hip_stream, double us[2] /* host */);

/*
 * Measurement aid, not a step of the path: a plain streaming read of device memory (16-byte
 * nontemporal loads, `n_workgroups` workgroups of 256 threads, each reading a contiguous
 * slice), timed with HIP events on `hip_stream` (synchronises).  Launch i reads the
 * `pass_bytes` bytes at offset (i mod floor(buf_bytes / pass_bytes)) * pass_bytes of `buf`, so
 * that with a buffer of several passes no launch finds an earlier one's bytes in the 256 MB
 * Infinity Cache.  What it reaches for a kernel's own byte count and launch shape is the rate
 * the machine leaves for that kernel; the published HBM peak stays the roofline's `peak`.
 * pass_bytes: a positive multiple of n_workgroups * 4096, at most buf_bytes; buf 16-byte
 * aligned.  us[0] = mean, us[1] = minimum microseconds per launch over `iters` after `warmup`.
 * Allocates and frees a few bytes of device memory (the sink that keeps the loads alive).
 */
TAPER_API int taper_stream_read_probe(taper_ctx *ctx, const void *buf /* device */, int64_t buf_bytes, int64_t pass_bytes,
                            int n_workgroups, int warmup, int iters, void *hip_stream, double us[2] /* host */);

/*
 * KV append: the step before attention in a decode loop.  The token a sequence
 * generated in the previous step becomes part of its context: its key and value
 * rows are written into the sequence's last private segment, right after that
 * segment's last token.  When the segment's pages are full (its length is a
 * multiple of page_size, 0 included) the token opens a new page, which the
 * caller must already have entered in the block table -- this is the only
 * moment a branch's memory grows (paper App. C "Memory accounting":
 * dM(j) = blocks(branch-local tokens), 0 for a branch that has produced nothing).
 *
 * taper_append_slots (host, integers only): slot[s] = page * page_size + token
 * where sequence s's next token goes, and opens_page[s] (may be NULL) = 1 when
 * that token is the first of a page.  Same batch arrays as
 * taper_plan_build_segments, lengths BEFORE the append.  TAPER_ELEN when a row
 * has no entry for the page, TAPER_EBLOCK when the entry is outside the pool,
 * TAPER_EINVAL when a sequence has no private segment.
 *
 * taper_kv_append: k_new, v_new bf16 [n_seqs][n_kv_heads][head_dim] (device),
 * slots int64 [n_seqs] (device), kv_pages the pool (device, written).  Enqueues
 * one kernel on hip_stream; allocates nothing, does not synchronise.  Slots must
 * be distinct.
 *
 * taper_branch_blocks: blocks(L) = ceil(L / page_size), the pages a branch with L
 * branch-local tokens occupies.
 */
TAPER_API int taper_append_slots(int n_seqs, const int32_t *block_table /* host */, int bt_row_stride,
                                 const int32_t *prefix_len /* host */, const int32_t *seg_start /* host */,
                                 const int32_t *seg_len /* host */, int page_size, int64_t n_pool_pages,
                                 int64_t *slots /* host, out */, int32_t *opens_page /* host, out, may be NULL */);
TAPER_API int taper_kv_append(taper_ctx *ctx, int n_seqs, const void *k_new /* device */, const void *v_new /* device */,
                              const int64_t *slots /* device */, void *kv_pages /* device */, void *hip_stream);
TAPER_API int64_t taper_branch_blocks(int64_t branch_local_tokens, int page_size);

TAPER_API const char *taper_strerror(int status);
TAPER_API const char *taper_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TAPER_ATTN_H */
