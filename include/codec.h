/*
 * codec.h - C ABI of the prefix-shared decode-attention library for MI355X (gfx950).
 *
 * The library computes, for a batch of decode requests whose contexts form a
 * forest of shared KV-cache nodes, out[r, hq, :] = softmax(scale * q[r, hq] . K_r^T) V_r
 * where K_r, V_r are the KV rows of the nodes on request r's prefix path,
 * concatenated root to leaf (paper Sec. 2.2 Eq. 1-2 and Sec. 4.1).  Each node's
 * KV rows are read from HBM once for the queries of all requests below the
 * node (partial attention computation, Alg. 2), and the per-node partial
 * results are merged per query (partial output reduction, Alg. 3; executor,
 * Alg. 4).  A host-side planner estimates per-node cost from a profiled table,
 * divides long nodes along the KV dimension and schedules the pieces onto
 * persistent workgroups (Sec. 5, Eq. 3-7).
 *
 * Conventions
 *  - Every function returns a status (0 = CODEC_OK, negative = error) unless
 *    stated otherwise; nothing throws or aborts; output parameters are left
 *    untouched on error.
 *  - "host" pointers are ordinary memory, borrowed for the duration of the
 *    call only.  "device" pointers are HIP device memory owned by the caller
 *    (e.g. PyTorch tensors); the library allocates no device memory.
 *  - Strides and offsets are in elements unless a name says bytes.
 *  - Query head hq uses KV head hq / (num_q_heads / num_kv_heads).
 */
#ifndef CODEC_H
#define CODEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CODEC_OK = 0,
    CODEC_ERR_INVALID_ARGUMENT = -1,    /* null pointer, non-positive count, bad option        */
    CODEC_ERR_INVALID_TREE = -2,        /* bad parent/req_node index, cycle, empty node, short page list */
    CODEC_ERR_UNSUPPORTED = -3,         /* head_dim not 64/128/256, unknown dtype, page size, group size */
    CODEC_ERR_WORKSPACE_TOO_SMALL = -4,
    CODEC_ERR_HIP = -5,                 /* a HIP runtime call failed                           */
    CODEC_ERR_NOT_UPLOADED = -6,        /* decode called before codec_plan_upload              */
    CODEC_ERR_OUT_OF_MEMORY = -7        /* host allocation failed                              */
};

enum { CODEC_DTYPE_FP16 = 0, CODEC_DTYPE_BF16 = 1 };

typedef struct codec_plan codec_plan_t;         /* opaque, library-owned, immutable after create */

/* Head layout (MHA / GQA / MQA; Sec. 6 "supports MHA, MQA and GQA"). */
typedef struct {
    int32_t num_q_heads;
    int32_t num_kv_heads;       /* must divide num_q_heads; group = ratio, 1..64        */
    int32_t head_dim;           /* 128; or 64 or 256, which run in the task shape for few
                                   rows only: group <= 16, query sets are tiled 32 (64
                                   channels) or 16 (256 channels) rows at a time (max_rows
                                   is capped), so a shared node is read once per tile, the
                                   repeats from cache                                   */
    int32_t dtype;              /* CODEC_DTYPE_*: type of q, K, V and out               */
    int32_t page_size;          /* tokens per KV page, a power of two, 16..4096         */
    float   scale;              /* softmax scale, 1/sqrt(head_dim) in Eq. 1             */
} codec_head_config;

/*
 * KV-cache forest (Sec. 4.1): node i holds node_len[i] >= 1 tokens that follow
 * the tokens of parent[i]; parent[i] = -1 makes i a child of the virtual root
 * that joins unrelated prefixes.  Request r's context ends with node
 * req_node[r] (a leaf or an internal node).  Node i owns the whole pages
 * page_ids[node_page_off[i] .. node_page_off[i+1]) and fills them in order, so
 * only its last page may be partly used.  All arrays are host memory.
 *
 * Visibility masks (Sec. 4.1: a position that is not visible to a query scores
 * -inf and contributes nothing; multi-token decoding, e.g. the verification of
 * tree-structured drafts).  A request is one query token.  It may carry a mask
 * over the tokens of the LAST node of its path: with the drafted tokens of a
 * sequence stored in one node, the query of a drafted token ends at that node
 * and sees, of its tokens, itself and the drafted tokens before it on its
 * branch; every token of the other nodes on its path is visible.
 * req_mask_off == NULL: no masks.  Else request r owns the 32-bit words
 * req_mask[req_mask_off[r] .. req_mask_off[r+1]): none (it sees everything), or
 * exactly one word per 32 tokens of node req_node[r], bit t % 32 of word t / 32
 * saying whether it sees token t; it must see at least one token of that node
 * (CODEC_ERR_INVALID_TREE otherwise).  A node that ends a masked request is not
 * divided along KV, and its queries are tiled 16 rows at a time; masks need
 * num_q_heads / num_kv_heads <= 16 (CODEC_ERR_UNSUPPORTED otherwise).
 */
typedef struct {
    int32_t        num_nodes;
    const int32_t *parent;          /* [num_nodes]      */
    const int32_t *node_len;        /* [num_nodes]      */
    int32_t        num_requests;
    const int32_t *req_node;        /* [num_requests]   */
    const int32_t *node_page_off;   /* [num_nodes + 1]  */
    const int32_t *page_ids;        /* [node_page_off[num_nodes]] */
    const int32_t  *req_mask_off;   /* NULL, or [num_requests + 1], ascending from 0 */
    const uint32_t *req_mask;       /* [req_mask_off[num_requests]] */
} codec_tree;

/*
 * Profiled cost table C_est (Sec. 5.2, Eq. 6; Table 2 is such a table):
 * cost[i * num_len_points + j] is the measured cost, in any integer unit, of
 * one workgroup running partial attention on row_grid[i] query rows (requests
 * x heads of one group) against len_grid[j] tokens.  Grids ascend strictly;
 * costs are > 0.  Between grid points the planner interpolates bilinearly in
 * integers (round half up); below the grid it clamps, above it continues the
 * last segment linearly.
 */
typedef struct {
    int32_t        num_row_points;
    int32_t        num_len_points;
    const int32_t *row_grid;
    const int32_t *len_grid;
    const int64_t *cost;
} codec_cost_table;

typedef struct {
    int32_t num_slots;      /* m of Eq. 3: persistent workgroups per KV head; 0 = as many as run at once:
                               256 / num_kv_heads if a task holds more than 16 rows of 128 channels, else
                               512 / num_kv_heads                                                   */
    int32_t split_align;    /* KV slices start on multiples of this many tokens; a multiple of
                               max(32, page_size); 0 = 256                                          */
    int32_t max_rows;       /* most query rows (requests x group) one task may hold, 1..256,
                               >= group; 0 = 256.  Larger query sets are cut into row tiles.       */
    int32_t share;          /* 1 = prefix-shared plan; 0 = flat baseline: every request gets its
                               own tasks for every node on its path, nothing shared across requests;
                               2 = whichever of up to four plans has the lowest estimated makespan:
                               the prefix-shared plan with row tiles of max_rows, with row tiles of
                               half that (if more than 16 rows), with row tiles of at most 16 rows
                               (query-dimension splits, b_q > 1 in the terms of Sec. 5.1; the last
                               one fits the narrow kernel variant) and the flat plan; ties go to the
                               earlier one.  The plan view reports the share and max_rows that won. */
    const codec_cost_table *cost;   /* NULL = built-in table of the kernel variant the plan needs     */
    int32_t fixed_slices;   /* 0 = the paper's adaptive division (Eq. 4-5 and the grid search);
                               n > 0 = the naive strategy it is compared with (Sec. 7, impact of
                               division granularity): every node is cut evenly into n slices (fewer
                               when the node is too short), then scheduled the same way            */
    int32_t schedule;       /* 0 = static: slot s runs the task list the greedy schedule gave it (Eq. 3's
                               assignment, as the paper executes it); 1 = run-time queue: the same tasks
                               in the same longest-first order, but a workgroup takes the next entry of
                               the queue when it has finished one, so that errors of the cost estimate
                               do not leave workgroups idle.  The first num_slots entries go to the
                               workgroups they would go to anyway; runs of short tasks form one entry.
                               The queue keeps two counters per KV head in the plan's device metadata:
                               one launch of a plan at a time; 2 = the library chooses: the queue if it
                               has at least six entries per slot (measured on irregular forests: with
                               that many the queue is 3-6 % faster, with few it changes nothing), else
                               static.  The plan view reports the schedule in use (0 or 1)           */
    int32_t fused;          /* 0 = Alg. 4 in two launches (partial attention, then reduction); 1 = one
                               launch: the workgroup whose task completes a request's set of partial
                               results (the last to arrive, counted per request and KV head in the
                               plan's device metadata) reduces them itself (the single-launch form
                               of the parallel reduction of Sec. 4.3, for trees whose step time is
                               of the order of a kernel launch); 2 = the library chooses: one launch
                               if the estimated makespan is below 40000 cost units (40 us with the
                               built-in tables) and the batch has at most 64 query rows per KV head
                               (one workgroup may be the last for all of them).  Only codec_decode_attention
                               (and its static variant) fuse; the two phase calls stay separate.  As
                               with the run-time queue, launches of one plan must not overlap.  The
                               plan view reports 0 or 1                                             */
    int32_t extensions;     /* 0 = the solver of Sec. 5.1 as printed: slice counts bounded by
                               ceil(C_est / cost_l) (Eq. 5), one node-by-node pass of the grid search.
                               Bits add this library's own extensions of it (CODEC_PLAN_EXT_*)       */
} codec_plan_options;

/*
 * Extensions of the Sec. 5.1 solver (not in the paper; each measured against the printed solver):
 *  CODEC_PLAN_EXT_SLACK     a node whose cost is at least cost_l / 4 may take one slice more than
 *                           the bound of Eq. 5 (lets a few nodes of 0.3 .. 1 average loads pack evenly)
 *  CODEC_PLAN_EXT_DIAGONAL  after the node-by-node pass the search also evaluates nine points on
 *                           the diagonal of the grid (every node at its Eq. 5 quotient for a common
 *                           target cost_l * (1 + k/8), k = 0 .. 8) and keeps the best point seen
 */
enum { CODEC_PLAN_EXT_SLACK = 1, CODEC_PLAN_EXT_DIAGONAL = 2 };

/* One work item of the division problem: a node (or a row tile of it) with its queries. */
typedef struct {
    int32_t node;
    int32_t q_off;          /* first entry of this item's requests in node_q                      */
    int32_t n_req;          /* requests in the item; rows = n_req * group                         */
    int32_t rows;
    int32_t len;            /* tokens of the node                                                 */
    int32_t ub;             /* most KV slices the search may give the item: the bound of Eq. 5,
                               ceil(cost / cost_l), one more under CODEC_PLAN_EXT_SLACK for an item
                               of at least cost_l / 4, as a count of aligned slices                  */
    int32_t b;              /* chosen number of KV slices b_k                                     */
    int32_t reserved;
    int64_t cost;           /* C_est(rows, len)                                                   */
} codec_item;

/* One partial-attention task: a KV slice of an item. */
typedef struct {
    int32_t item;
    int32_t node;
    int32_t kv_begin;       /* first token of the slice inside the node                           */
    int32_t kv_len;
    int32_t q_off;
    int32_t n_req;
    int32_t part_row_base;  /* first of the task's n_req * group partial rows                     */
    int32_t slot;           /* workgroup slot the task is scheduled on                            */
    int64_t cost;           /* C_est(rows, kv_len)                                                */
} codec_task;

/*
 * Read-only host view of a plan; pointers stay valid until codec_plan_destroy.
 * node_q lists, per node, the requests whose path contains it (ascending);
 * slot s runs tasks slot_tasks[slot_off[s] .. slot_off[s+1]) in that order;
 * request r merges the partials whose first rows are
 * req_part[req_part_off[r] .. req_part_off[r+1]) (root to leaf, slices in order).
 */
typedef struct {
    int32_t           num_items;
    const codec_item *items;
    int32_t           num_tasks;
    const codec_task *tasks;
    int32_t           num_slots;
    const int32_t    *slot_off;
    const int32_t    *slot_tasks;
    int32_t           num_nodes;
    const int32_t    *node_q_off;
    const int32_t    *node_q;
    int32_t           num_requests;
    const int32_t    *req_part_off;
    const int32_t    *req_part;
    int64_t           cost_l;       /* lower bound of the makespan from Eq. 4                     */
    int64_t           makespan;     /* estimated cost of the most loaded slot                     */
    int32_t           part_rows;    /* partial rows per KV head                                   */
    int32_t           split_align;
    int32_t           max_rows;
    int32_t           share;
    int32_t           schedule;
    int32_t           fused;
    int32_t           num_entries;  /* run-time queue (also built for static plans): entry e holds tasks */
    const int32_t    *queue_off;    /* queue_tasks[queue_off[e] .. queue_off[e+1]); entries in order of  */
    const int32_t    *queue_tasks;  /* decreasing cost of their first task                               */
} codec_plan_view;

/*
 * Layout of the K and V page pools (both pools share it): element (page, slot, kv head, c)
 * lives at page * page_stride + slot * token_stride + kv head * head_stride + c.  The head_dim
 * elements of a head are contiguous; strides are multiples of 8 elements.  num_pages is
 * the pool size; every page id of the plan must be below it.
 */
typedef struct {
    int64_t num_pages;
    int64_t page_stride;
    int64_t token_stride;
    int64_t head_stride;
} codec_kv_layout;

/*
 * Build a plan (Sec. 5): index the forest (per-node query sets, per-request
 * paths; Sec. 4.1), estimate costs (Eq. 6-7), bound and choose the number of
 * KV slices of every node (Eq. 4-5, grid search) and schedule the slices
 * longest-first onto num_slots slots (Eq. 3).  Host only: no HIP call is made.
 * All inputs are host memory and are copied.  *out receives the plan.
 */
int codec_plan_create(const codec_tree *tree, const codec_head_config *head,
                      const codec_plan_options *options, codec_plan_t **out);

/* Frees a plan (host memory only).  NULL is accepted. */
int codec_plan_destroy(codec_plan_t *plan);

/* Fills *view with pointers into the plan's own host arrays. */
int codec_plan_export(const codec_plan_t *plan, codec_plan_view *view);

/*
 * Carry a plan over to the next decoding steps without planning again.  The
 * paper divides tasks only every few decoding steps (Implementation section,
 * task division module) while every step appends tokens to the requests' last
 * nodes; in between, the division and the slot assignment are kept: every slice
 * keeps its boundaries, the last slice of a node takes up the node's change in
 * length, costs and the estimated makespan (see codec_plan_export) are
 * recomputed.  The forest itself (parents, requests) must be the one the plan
 * was created for; node_len[num_nodes], node_page_off[num_nodes + 1] and
 * page_ids[node_page_off[num_nodes]] are host arrays with the meaning they have
 * in codec_tree and are copied.  Host only.  Visibility masks are kept as they
 * are: a node that ends a masked request must keep its length.
 *
 * The device copy of the metadata becomes stale: codec_plan_device_bytes may
 * have grown (longer page lists) and codec_plan_upload must be called again
 * before the next launch (launches return CODEC_ERR_NOT_UPLOADED until then).
 * Pointers obtained from codec_plan_export before the call are invalid after it.
 *
 * Errors (the plan is left unchanged): CODEC_ERR_INVALID_TREE for a length
 * below 1, a page list shorter than its node or a negative page id;
 * CODEC_ERR_INVALID_ARGUMENT for NULL arrays or a length that would leave a
 * node's last slice empty (the node shrank below the start of that slice: plan
 * again).
 */
int codec_plan_refresh_lengths(codec_plan_t *plan, const int32_t *node_len,
                               const int32_t *node_page_off, const int32_t *page_ids);

/*
 * C_est(rows, len) of Eq. 6 on `table`; returns the cost, or a negative status.  NULL = the
 * built-in table of the kernel variant a task of `rows` rows needs (wide above 16 rows).
 */
int64_t codec_cost_estimate(const codec_cost_table *table, int32_t rows, int32_t len);

/*
 * The built-in cost tables (static storage), profiled on an MI355X in ns per task: wide != 0 for
 * plans that hold a task of more than 16 query rows, wide == 0 for the others (the kernel runs such
 * plans with a different workgroup shape, see num_slots).
 */
const codec_cost_table *codec_default_cost_table(int32_t wide);

/* Bytes of device memory the plan's task lists and indexes need. */
size_t codec_plan_device_bytes(const codec_plan_t *plan);

/*
 * Copies the plan's device-side metadata into `device_meta` (device memory,
 * >= codec_plan_device_bytes, 256-byte aligned, caller-owned, must outlive all
 * decode calls on this plan) on `stream` (a hipStream_t, may be NULL) and
 * remembers the pointer.  Call once per plan before decoding.  With
 * schedule = 1 the kernels keep the queue's counters in this memory (zero after
 * the upload, zero again after every completed launch): launches of one plan
 * must not overlap, and a launch that was aborted leaves them undefined (upload
 * again).
 */
int codec_plan_upload(codec_plan_t *plan, void *device_meta, size_t device_meta_bytes, void *stream);

/* Bytes of scratch (partial outputs with their softmax statistics) one decode call needs. */
size_t codec_plan_workspace_bytes(const codec_plan_t *plan);

/*
 * One decode-attention step (Alg. 4): partial attention for every scheduled
 * task, then per-query reduction, enqueued on `stream`; returns without
 * synchronising.
 *   q        device [num_requests][num_q_heads][head_dim], dtype of the plan, 16-byte aligned
 *   k_pages, v_pages   device page pools, laid out by `layout`, 16-byte aligned
 *   out      device [num_requests][num_q_heads][head_dim], same dtype
 *   workspace  device scratch, >= codec_plan_workspace_bytes, 256-byte aligned;
 *              contents are overwritten; calls sharing a workspace must not overlap
 */
int codec_decode_attention(const codec_plan_t *plan, const void *q,
                           const void *k_pages, const void *v_pages,
                           const codec_kv_layout *layout, void *out,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * The two phases of Alg. 4 on their own, for callers that time or overlap them:
 * codec_partial_attention runs the scheduled partial attention tasks and fills
 * `workspace`; codec_partial_reduction merges the partials in `workspace` into
 * `out`.  Same arguments, checks and stream semantics as codec_decode_attention,
 * which is exactly the first followed by the second.
 */
int codec_partial_attention(const codec_plan_t *plan, const void *q,
                            const void *k_pages, const void *v_pages,
                            const codec_kv_layout *layout,
                            void *workspace, size_t workspace_bytes, void *stream);
int codec_partial_reduction(const codec_plan_t *plan, const void *workspace,
                            size_t workspace_bytes, void *out, void *stream);

/*
 * codec_decode_attention for callers that cannot allocate device memory and hold no workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same
 * two kernels run with the partial results in a scratch array of the library's own (static device
 * memory, CODEC_STATIC_SCRATCH_BYTES = 64 MiB per GPU, held until the process ends); the call
 * allocates and frees nothing.  q, k_pages, v_pages, layout, out and stream are those of
 * codec_decode_attention; the plan must have been uploaded (codec_plan_upload, which is also where
 * the one-off kernel attributes are set) with the device it was uploaded to current.
 * Errors: CODEC_ERR_WORKSPACE_TOO_SMALL if codec_plan_workspace_bytes(plan) exceeds the array
 * (codec_last_error_message names both sizes); otherwise as codec_decode_attention.
 * Every call on a GPU uses that GPU's one array, which keeps the previous call's contents (nothing in
 * it has to start at zero: every partial row a call reads, it has written first): calls that
 * overlap on one GPU, on any streams, race.
 */
#define CODEC_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int codec_decode_attention_static(const codec_plan_t *plan, const void *q,
                                  const void *k_pages, const void *v_pages,
                                  const codec_kv_layout *layout, void *out, void *stream);
size_t codec_static_scratch_bytes(void);       /* CODEC_STATIC_SCRATCH_BYTES of the built library */

/*
 * Measurement support (no part of the method): a read-only streaming kernel that gives the HBM read
 * rate this machine reaches, for pricing the attention kernel against something measured beside the
 * vendor's 8 TB/s.  Reads `bytes` (a power of two, >= 4096) of device memory at `buffer` (16-byte
 * aligned) once, 16 bytes per lane, with `workgroups` workgroups of 256 threads taking 4 KB chunks
 * round-robin; pattern 0 = chunks in address order, 1 = in a scattered order (the pattern of a paged
 * pool with 4 KB page-heads); nontemporal != 0 = loads with the streaming hint.  `sink` is device
 * memory of `workgroups` 32-bit words (written practically never; keeps the loads alive).
 * Enqueues on `stream` and returns; the caller times it.
 */
int codec_stream_read_probe(const void *buffer, size_t bytes, int32_t pattern, int32_t nontemporal,
                            int32_t workgroups, void *sink, void *stream);

/* Static, human-readable name of a status code. */
const char *codec_status_string(int status);

/*
 * Text of the HIP runtime's error for the calling thread's most recent CODEC_ERR_HIP
 * (the failing call and hipGetErrorString of its result); "" if there was none.
 * The pointer stays valid until the thread's next failing call.
 */
const char *codec_last_error_message(void);

#ifdef __cplusplus
}
#endif
#endif /* CODEC_H */
