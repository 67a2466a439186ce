/*
 * tokenlake.h -- C ABI of the MI355X (gfx950) segment-level prefix-attention library.
 *
 * The library implements the data-plane compute of TokenLake's cache-aware operation
 * (paper Section 3.2 "Interfaces": `query` returns the attention output of the query
 * tensor over the prefix-cache pool, `put` stores new KV; Section 4, first paragraph:
 * segments are independent, each yields a partial output and a normalizer, and the
 * final output is their combination; Section 2.1: prefix attention and the new tokens'
 * self-attention are reduced together).
 *
 * Conventions
 *  - Every call returns a tl_status (0 = TL_OK, negative = error).  Nothing throws or
 *    aborts across this boundary; tl_last_error() gives a per-thread message.
 *  - "host" pointers are ordinary CPU memory, read during the call only.
 *    "device" pointers are HIP device memory owned by the caller unless stated otherwise;
 *    they must stay valid until the stream work enqueued by the call has completed.
 *  - Compute calls enqueue kernels on `stream` (a hipStream_t passed as void*, NULL = the
 *    default stream) and return without synchronising.
 *    tl_segment_attn, tl_causal_block, tl_merge and tl_fused_attn enqueue nothing but
 *    kernels, except that the first call that uses a plan makes the plan's device copy (one
 *    hipMalloc, one asynchronous copy on `stream`) and the first tl_segment_attn after an
 *    adopt or evict uploads the pool's fill table (one asynchronous copy): run one step
 *    eagerly before capturing a step into a HIP graph.
 *  - A pool, and the plans made from it, belong to one host thread at a time: calls on the
 *    same pool or plan from several threads need the caller's own lock (the id table, the
 *    use stamps and the lazily made device copies are plain host state).  Different pools
 *    are independent.  Compute calls on one stream run in order; the same plan may be used
 *    on several streams once its first call has returned.
 *  - With a plan of zero new tokens the compute calls return TL_OK at once and look at no
 *    other argument (empty tensors have null pointers).
 *  - A plan holds slot numbers and fills as they were when it was built.  Any change to the
 *    pool's slots afterwards (tl_pool_put of a new id, tl_pool_append, tl_pool_append_batch,
 *    tl_pool_adopt, tl_pool_evict_lru) makes it stale: tl_segment_attn and tl_fused_attn then
 *    return TL_EINVAL and enqueue nothing; build a new plan (Section 3.2: plans are made per
 *    iteration).  tl_pool_release and a put of a resident id change no slot and keep plans valid.
 *    A plan may outlive its pool only to be destroyed or read back (info, export, hot slots).
 *  - All tensors are dense, row-major, bf16 = 16-bit brain float bit patterns.
 *  - head_dim must be 128; q_heads must be a multiple of kv_heads, at most 32 times it; seg_len must
 *    be a multiple of 64.  Anything else is TL_EINVAL.
 *  - The normalizer is the natural-log log-sum-exp of the scaled scores.  A row with no
 *    keys has O = 0 and LSE = -inf.
 */
#ifndef TOKENLAKE_H_
#define TOKENLAKE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t tl_status;
enum {
  TL_OK = 0,
  TL_EINVAL = -1,    /* bad argument (null pointer, size, unsupported shape)          */
  TL_ENOMEM = -2,    /* host or device allocation failed                              */
  TL_EFULL = -3,     /* no free slot in the pool                                      */
  TL_ENOTFOUND = -4, /* segment id not resident in the pool                           */
  TL_EHIP = -5       /* a HIP runtime call failed (no device, launch error, ...)      */
};

/* Text for a status code (static storage). */
const char* tl_status_str(tl_status s);
/* Message of the last failing call on this thread (static thread-local storage). */
const char* tl_last_error(void);

/* ------------------------------------------------------------------------------------
 * Segment pool (paper Section 3.1: prefix caches are split into fixed-size segments kept in
 * per-GPU cache slots; Section 1 / 4: one copy per segment -- deduplication).
 *
 * Slot s holds K and V as [seg_len, kv_heads, head_dim] bf16 each, at
 *   k_dev + s * seg_len * kv_heads * head_dim   (same for v_dev).
 * A slot has `fill` valid tokens (1..seg_len); tokens at or beyond fill do not exist for
 * attention.  The pool object lives on the host; it owns the id->slot table, the per-slot
 * fill / reference count / last-use stamp, and a device mirror of fill[].
 * ------------------------------------------------------------------------------------ */
typedef struct tl_pool tl_pool;

/* k_dev/v_dev: device, [n_slots, seg_len, kv_heads, head_dim] bf16 each, caller-owned; or
 * both NULL, then the library allocates them (and frees them in tl_pool_destroy).
 * Makes no HIP call when k_dev/v_dev are given (device state is set up on first use). */
tl_status tl_pool_create(tl_pool** out, int32_t n_slots, int32_t seg_len, int32_t kv_heads,
                         int32_t head_dim, void* k_dev, void* v_dev);
tl_status tl_pool_destroy(tl_pool* pool);

/* `put` (Section 3.2): store one segment.  k_src_dev/v_src_dev: device,
 * [fill, kv_heads, head_dim] bf16.  If the id is already resident nothing is copied, its
 * reference count goes up and *slot_out is the existing slot (deduplication).  Otherwise
 * the segment goes to want_slot (must be free) or, with want_slot = -1, to the
 * lowest-numbered free slot; tokens [fill, seg_len) of the slot are zeroed.
 * Errors: TL_EFULL, TL_EINVAL (fill outside 1..seg_len, slot taken or out of range). */
tl_status tl_pool_put(tl_pool* pool, uint64_t segment_id, const void* k_src_dev, const void* v_src_dev,
                      int32_t fill, int32_t want_slot, int32_t* slot_out, void* stream);

/* Append the K/V of n_rows new tokens to a chain of private segments (Section 3.2: the KV of
 * the tokens just computed is `put` into the pool and is prefix cache for the next turn).
 * Rows go, in order, first into the slot of tail_id from its current fill up to seg_len
 * (has_tail = 0: the chain has no partly filled tail, tail_id is ignored), then into new
 * segments new_ids[0..n_new) in order, seg_len rows each, the last possibly partly filled
 * (its remaining tokens are zeroed).  Each new id takes the lowest-numbered free slot.
 * k_rows_dev/v_rows_dev: device, [n_rows, kv_heads, head_dim] bf16.  new_ids: host [n_new];
 * n_new must be exactly ceil(max(0, n_rows - room in the tail) / seg_len).
 * new_slots_out: host [n_new] or NULL.  One kernel launch per 128 destination slots.
 * The tail must hold exactly one reference (a segment somebody else also uses does not grow).
 * Nothing is written or registered on error: TL_ENOTFOUND (tail not resident), TL_EINVAL
 * (tail shared, wrong n_new, id repeated or already resident), TL_EFULL. */
tl_status tl_pool_append(tl_pool* pool, int32_t has_tail, uint64_t tail_id, const uint64_t* new_ids, int32_t n_new,
                         const void* k_rows_dev, const void* v_rows_dev, int32_t n_rows, int32_t* new_slots_out,
                         void* stream);

/* tl_pool_append for n_chains chains in one call (the sessions of a batch after a turn): chain c
 * appends rows [row_ptr[c], row_ptr[c+1]) of k_rows_dev/v_rows_dev, first into the slot of
 * tail_ids[c] if has_tail[c] is non-zero, then into new segments new_ids[new_ptr[c] .. new_ptr[c+1]).
 * has_tail, tail_ids (may be NULL if no chain has a tail): host [n_chains]; new_ptr, row_ptr:
 * host [n_chains + 1], starting at 0, non-decreasing; new_slots_out: host [new_ptr[n_chains]] or
 * NULL.  Chains are served in order, each new id taking the lowest-numbered free slot, so the
 * result equals that of n_chains single calls; the rows of all chains go out in one kernel
 * launch per 128 destination slots.  Every chain is validated before anything is written or
 * registered: errors as for tl_pool_append, and TL_EINVAL if two chains name the same tail. */
tl_status tl_pool_append_batch(tl_pool* pool, int32_t n_chains, const int32_t* has_tail, const uint64_t* tail_ids,
                               const int32_t* new_ptr, const uint64_t* new_ids, const int32_t* row_ptr,
                               const void* k_rows_dev, const void* v_rows_dev, int32_t* new_slots_out, void* stream);

/* Register segments whose KV the caller has already written into the pool memory
 * (no copy; the slots' tails are left as they are).  ids/slots/fills: host, [n].
 * Same id twice or slot taken -> TL_EINVAL, nothing is registered. */
tl_status tl_pool_adopt(tl_pool* pool, const uint64_t* ids, const int32_t* slots, const int32_t* fills,
                        int32_t n, void* stream);

/* Drop one reference.  A segment with zero references stays resident (it can still be
 * looked up and attended to) until tl_pool_evict_lru removes it.  TL_ENOTFOUND for an
 * unknown id, TL_EINVAL if the count is already zero. */
tl_status tl_pool_release(tl_pool* pool, uint64_t segment_id);

/* Free the slot of the least recently used segment among those with zero references
 * (Section 4.3: eviction by last access time).  A segment is "used" when it is put,
 * adopted, or named by a plan.  *evicted_id receives its id; TL_ENOTFOUND if no segment
 * is evictable. */
tl_status tl_pool_evict_lru(tl_pool* pool, uint64_t* evicted_id);

/* The pool's prefix tree (Section 3.1: a global prefix tree indexes the segments; Section 3.2:
 * `get_prefix_tree` hands it to the scheduler; Section 4.3: a segment is accessed only when its
 * prefix is, so load concentrates near the root and heavy hitters are found from the root without
 * walking the whole tree).  The tree lives in the pool across batches: tl_plan_create walks every
 * request's list from the root, makes the nodes that are missing -- a node is a segment id under a
 * given parent; the same id under two prefixes is two nodes of one slot -- and adds the request's
 * new tokens to the load of every node on the way, so a node is never more loaded than its parent.
 * tl_pool_evict_lru removes the evicted segment's nodes with everything below them.  Lists that
 * follow no tree (the same segments in ever new orders) make new nodes with every batch: when the
 * tree has grown beyond 16 nodes per slot of the pool, the next tl_plan_create clears it and the
 * cumulative loads start over.
 *
 * tl_pool_hot_segments: up to max_n nodes by decreasing cumulative load (equal loads: the older node
 * first, so a parent precedes its children), found by a best-first search from the root that looks
 * only at the children of the nodes it returns.  ids_out: host [max_n]; loads_out (new tokens that
 * attended to the node), depths_out (0 = first segment of a prefix): host [max_n] or NULL.
 *
 * tl_pool_prefix_tree: the tree in level order from the root, at most max_nodes nodes: segment id,
 * position of the parent in the same output (-1 = child of the root; a parent always comes first)
 * and cumulative load.  *n_total_out (may be NULL) = nodes in the whole tree. */
tl_status tl_pool_hot_segments(const tl_pool* pool, int32_t max_n, uint64_t* ids_out, int64_t* loads_out,
                               int32_t* depths_out, int32_t* n_out);
tl_status tl_pool_prefix_tree(const tl_pool* pool, int32_t max_nodes, uint64_t* ids_out, int32_t* parents_out,
                              int64_t* loads_out, int32_t* n_out, int32_t* n_total_out);

/* segment_id -> slot for n ids (host arrays); -1 for an id that is not resident.
 * Never fails on a miss.  Bit-exact integer work. */
tl_status tl_pool_lookup(const tl_pool* pool, const uint64_t* ids, int32_t n, int32_t* slots_out);
/* Valid tokens of n slots (host arrays); 0 for a free slot. */
tl_status tl_pool_fills(const tl_pool* pool, const int32_t* slots, int32_t n, int32_t* fills_out);
/* Counters: slots in use. */
tl_status tl_pool_used(const tl_pool* pool, int32_t* n_used);

/* Copy the listed slots, whole (seg_len tokens each), to contiguous device buffers
 * k_out_dev/v_out_dev [n, seg_len, kv_heads, head_dim].  slots: host [n] (read before the call
 * returns).  Enqueued on `stream` (512 slots per launch); allocates nothing and does not wait.
 * For verification of slot addressing; bit-exact. */
tl_status tl_pool_gather(tl_pool* pool, const int32_t* slots, int32_t n, void* k_out_dev, void* v_out_dev,
                         void* stream);

/* ------------------------------------------------------------------------------------
 * Plan: the per-iteration control flow (Section 3.2: plans are generated for each batch
 * before the data plane runs).  Built on the host from each request's new-token range and
 * ordered segment-id list.  It resolves ids to slots, groups requests that share a run of
 * slots into one work item (a hot segment is then read once for all their query rows,
 * Section 4.3), splits long lists of decode requests into chunks (split-K), and lays out
 * the partial rows and the merge lists.
 *
 * Partial row p of out_partial/lse belongs to one (work item, token) pair; the causal self
 * block, if requested, owns rows [self_row_base, self_row_base + n_tokens).
 * ------------------------------------------------------------------------------------ */
typedef struct tl_plan tl_plan;

enum {
  TL_PLAN_SELF_BLOCK = 1, /* reserve partial rows for tl_causal_block and merge them   */
  TL_PLAN_NO_SHARING = 2, /* do not group requests: one item chain per request         */
  TL_PLAN_WALK_REPEATS = 8, /* a row-tile work item walks a slot once per occurrence in its list.
                             Default (flag absent): a slot that the list names m times is walked
                             once with weight m (exact: m equal keys contribute m exp(s) to the
                             numerator and the denominator alike)                          */
  TL_PLAN_FUSE_ROWS = 4,  /* requests that gain nothing from sharing a run of slots leave the
                             three-step path: one pass of tl_fused_attn over their whole slot
                             list and their own new tokens writes their final output.  These
                             are the requests with more than 16 query rows per kv head (new
                             tokens x q-heads per kv-head) that have no segment in common with
                             another request of the batch, or at least 512 such rows -- except,
                             in a batch of fewer row-tile workgroups than the GPU has CUs, those
                             whose lists are long enough (> 2048 tokens) to be cut along the
                             KV instead.  Such rows have a single partial, so nothing is
                             written to out_partial for them and tl_segment_attn /
                             tl_causal_block / tl_merge skip them.  Needs TL_PLAN_SELF_BLOCK. */
  TL_PLAN_FUSE_TAILS = 16 /* every request with more than 16 query rows per kv head (that
                             TL_PLAN_FUSE_ROWS, if also given, has not taken whole) is cut where its
                             list stops being shared: the runs it shares with other requests stay
                             work items of tl_segment_attn -- a hot segment is read once for all its
                             requesters' rows (Section 4.3) -- and the rest of its list together with
                             its own new tokens is one pass of tl_fused_attn, whose epilogue merges
                             the request's partial rows of those work items in and writes the final
                             output.  No causal tile, no partial of its own and no tl_merge for such
                             a request; tl_fused_attn must follow tl_segment_attn on the same stream
                             and be given the partial buffers.  (In a batch of fewer row-tile
                             workgroups than the GPU has CUs a private run longer than 2048 tokens is
                             cut along its KV instead, as without the flag.)  Needs
                             TL_PLAN_SELF_BLOCK; not with TL_PLAN_NO_SHARING. */
};

typedef struct tl_plan_info {
  int32_t n_req, n_tokens, q_heads, kv_heads;
  int32_t n_items;         /* work items of tl_segment_attn                              */
  int32_t n_partial_rows;  /* R: rows the caller must provide in out_partial / lse       */
  int32_t self_row_base;   /* first row of the self block, -1 without TL_PLAN_SELF_BLOCK */
  int32_t n_tiles;         /* MFMA row tiles (work items with many query rows)           */
  int32_t n_units;         /* split-K units (work items with <= 16 rows per kv head)     */
  int32_t n_causal_tiles;  /* row tiles of tl_causal_block (requests with two or more new tokens) */
  int32_t n_list_entries;  /* sum of request list lengths                                */
  int32_t n_merge_entries; /* sum over tokens of partials to merge                       */
  int64_t prefix_pairs;    /* sum over list entries of new_tokens(req) * fill(slot)      */
  int64_t self_pairs;      /* sum over requests of Lq (Lq + 1) / 2                       */
  int64_t unique_kv_tokens;/* valid tokens in the distinct slots the plan touches        */
  int32_t n_fused_tiles;   /* row tiles of tl_fused_attn (TL_PLAN_FUSE_ROWS)             */
  int32_t n_fused_tokens;  /* new tokens whose output tl_fused_attn writes               */
  int32_t n_single_tokens; /* requests with one new token (decode): their self block is one key,
                              written by a light kernel of tl_causal_block                */
  int64_t tile_pairs;      /* (query token, kv token) pairs the row-tile kernels compute: as
                              prefix_pairs over row-tile work, each distinct slot of a work
                              item's list counted once (unless TL_PLAN_WALK_REPEATS)       */
  int64_t item_pairs;      /* the part of prefix_pairs that tl_segment_attn's work items compute
                              (the rest belongs to tl_fused_attn's one-pass rows and tails)   */
  int32_t n_prior_rows;    /* partial rows of work items that tl_fused_attn merges in itself
                              (TL_PLAN_FUSE_TAILS), counted per (request, work item)           */
} tl_plan_info;

/* req_row_ptr: host [n_req+1], offsets of each request's new tokens in the batch's Q
 * (req_row_ptr[0] = 0, non-decreasing).  req_seg_ptr: host [n_req+1], offsets into seg_ids.
 * seg_ids: host, the ordered prefix of each request.  split_segments: list entries per
 * split-K chunk for items with few rows (0 = library default).  compute_units: the number
 * of CUs the plan fills (negative = 256, MI355X; at most 4096): a batch with fewer row-tile
 * workgroups than this gets KV-chunked work items instead of one-pass rows, and the default
 * split-K chunk is sized for it; 0 = never cut a row-tile item along its KV.
 * Errors: TL_ENOTFOUND if an id is not resident; TL_EINVAL on malformed arrays.
 * Makes no HIP call: the device copy of the plan is made by the first compute call that uses
 * it (one hipMalloc and one copy enqueued on that call's stream). */
tl_status tl_plan_create(tl_plan** out, const tl_pool* pool, int32_t q_heads, int32_t n_req,
                         const int32_t* req_row_ptr, const int32_t* req_seg_ptr, const uint64_t* seg_ids,
                         int32_t flags, int32_t split_segments, int32_t compute_units);
tl_status tl_plan_destroy(tl_plan* plan);
tl_status tl_plan_get_info(const tl_plan* plan, tl_plan_info* info);

/* Host copies of the plan's integer structure, for checking it (each pointer may be NULL
 * to skip; arrays must be large enough, sizes from tl_plan_info):
 *   item_row_base [n_items]     first partial row of the item
 *   item_tok_ptr  [n_items+1]   into item_tokens
 *   item_tokens   [..]          batch token index of each of the item's rows, in row order
 *   item_slot_ptr [n_items+1]   into item_slots
 *   item_slots    [..]          the item's ordered slot list
 *   merge_ptr     [n_tokens+1]  into merge_rows
 *   merge_rows    [n_merge_entries] partial rows to combine for each token            */
tl_status tl_plan_export(const tl_plan* plan, int32_t* item_row_base, int32_t* item_tok_ptr,
                         int32_t* item_tokens, int32_t* item_slot_ptr, int32_t* item_slots,
                         int32_t* merge_ptr, int32_t* merge_rows);
/* Heavy hitters of the batch (Section 4.3: load concentrates on segments near the root of the
 * prefix tree; they are found from the root without walking the whole tree and are the candidates
 * for replication).  The plan keeps the part of the pool's prefix tree that its requests walked,
 * each node with the new tokens of the requests that passed through it; this call returns up to
 * max_n of those nodes in order of decreasing load -- equal loads in order of first visit (requests
 * in order, lists front to back), so a parent precedes its children -- by a best-first search from
 * the root that looks only at the children of what it returns.  A segment that sits at several
 * tree positions (lists that name it under different prefixes, or twice) appears once per position.
 * slots_out: host [max_n] int32, the nodes' slots; loads_out: host [max_n] int64 or NULL. */
tl_status tl_plan_hot_slots(const tl_plan* plan, int32_t max_n, int32_t* slots_out, int64_t* loads_out, int32_t* n_out);

/* Sizes of the two variable-length arrays of tl_plan_export. */
tl_status tl_plan_export_sizes(const tl_plan* plan, int32_t* n_item_tokens, int32_t* n_item_slots);

/* ------------------------------------------------------------------------------------
 * Compute (Section 3.2 `query`; Section 4 first paragraph; Section 2.1).
 * ------------------------------------------------------------------------------------ */

/* Partial attention of every work item: for each of its query rows (token, q-head) the
 * softmax attention over the valid tokens of the item's slots, in list order:
 *   s_j = scale * <q, k_j>,  LSE = ln sum_j exp(s_j),  O = sum_j exp(s_j - LSE) v_j.
 * q_dev: device [n_tokens, q_heads, 128] bf16.
 * out_partial: device [n_partial_rows, q_heads, 128] fp32;  lse: device [n_partial_rows, q_heads] fp32.
 * Rows of the self block are not written by this call. */
tl_status tl_segment_attn(const tl_pool* pool, tl_plan* plan, const void* q_dev, float scale,
                          float* out_partial, float* lse, void* stream);

/* Causal self block of the new tokens: token i of a request attends to the request's new
 * tokens 0..i (inclusive).  k_new_dev/v_new_dev: device [n_tokens, kv_heads, 128] bf16.
 * Writes partial rows [self_row_base, self_row_base + n_tokens).  TL_EINVAL if the plan was
 * built without TL_PLAN_SELF_BLOCK. */
tl_status tl_causal_block(tl_plan* plan, const void* q_dev, const void* k_new_dev, const void* v_new_dev,
                          float scale, float* out_partial, float* lse, void* stream);

/* The whole path in one pass for the requests that TL_PLAN_FUSE_ROWS took out of the three
 * steps (paper Section 3.3: prefix attention and the new tokens' self-attention of a request
 * need not be separate passes when one engine holds both): each row tile walks the request's
 * pool tiles, then the new tokens up to its own rows, and writes the normalised output.
 * q_dev, k_new_dev, v_new_dev as in tl_causal_block.  out_dev: device [n_tokens, q_heads, 128],
 * bf16 if out_is_bf16 else fp32; lse_out: device [n_tokens, q_heads] fp32 or NULL.  Only the
 * fused requests' tokens are written; the other tokens of the same arrays are written by
 * tl_merge.  A plan without fused requests: nothing to do, TL_OK.
 * prior_partial / prior_lse: device, the out_partial / lse arrays that tl_segment_attn has written
 * for this plan earlier on the same stream; read only under TL_PLAN_FUSE_TAILS (the partial rows of
 * the shared runs above each one-pass tail, merged in by the epilogue with the rule of tl_merge);
 * may be NULL when the plan's n_prior_rows is 0, else TL_EINVAL. */
tl_status tl_fused_attn(const tl_pool* pool, tl_plan* plan, const void* q_dev, const void* k_new_dev,
                        const void* v_new_dev, float scale, const float* prior_partial, const float* prior_lse,
                        void* out_dev, int32_t out_is_bf16, float* lse_out, void* stream);

/* tl_fused_attn for callers that cannot allocate device memory (code under HIP graph capture set-up
 * rules, tight serving loops, harnesses that forbid hipMalloc): same arguments, same kernels, same
 * result bit for bit, but the plan's device-side work lists, which tl_fused_attn keeps in memory
 * it hipMalloc's on the plan's first use, are staged in a buffer that is part of the library's
 * device code (4 MiB per GPU, held until the process ends).  The call makes no hipMalloc, hipFree
 * or other allocating call: it looks up the buffer's address (once per device, on the first call
 * with that device current), enqueues one host-to-device copy of the work lists and the kernel on
 * `stream`.  TL_EINVAL if the plan's work lists exceed 4 MiB (the named workloads take 20-400 KB)
 * or the device index is 64 or more.  All calls on one GPU share the buffer, which keeps the last
 * call's contents: calls on one stream are ordered and safe; calls that overlap on one GPU (two
 * streams, two threads) race and must be serialised by the caller. */
tl_status tl_fused_attn_static(const tl_pool* pool, tl_plan* plan, const void* q_dev, const void* k_new_dev,
                               const void* v_new_dev, float scale, const float* prior_partial,
                               const float* prior_lse, void* out_dev, int32_t out_is_bf16, float* lse_out,
                               void* stream);

/* Exact recombination of each token's partials (Section 2.1: partial outputs and normalizers are
 * reduced into the final output; Section 4, first paragraph):
 *   M = max_j LSE_j, w_j = exp(LSE_j - M), O = sum_j w_j O_j / sum_j w_j, LSE = M + ln sum_j w_j.
 * out_partial / lse: device, the rows that tl_segment_attn and tl_causal_block wrote.
 * out_dev: device [n_tokens, q_heads, 128], bf16 if out_is_bf16 else fp32.
 * lse_out: device [n_tokens, q_heads] fp32, or NULL.  Tokens of one-pass requests are not written. */
tl_status tl_merge(tl_plan* plan, const float* out_partial, const float* lse, void* out_dev,
                   int32_t out_is_bf16, float* lse_out, void* stream);

/* Switch for tests (process-wide; both settings compute the same thing).  Returns TL_EINVAL for
 * an unknown knob or a value out of range.  Knob:
 *   "vread"   0 (default) = transposing LDS reads of V, 1 = scalar LDS reads. */
tl_status tl_set_option(const char* knob, int32_t value);

/* ------------------------------------------------------------------------------------
 * Analytic models (host arithmetic, no GPU work).  Units: seconds, bytes, flop/s, bytes/s,
 * tokens; 16-bit elements as in the paper.  d_q = q_heads * head_dim (flops and the query /
 * partial-output rows on the wire follow it), d_kv = kv_heads * head_dim (KV bytes follow it);
 * the paper's multi-head model has d_q = d_kv = d.  TL_EINVAL for non-positive sizes or rates,
 * negative latency or time, null outputs.
 * ------------------------------------------------------------------------------------ */
/* Section 4.1: T_comp = n_tokens * max(4 d_q / flops, 4 d_kv / mem_bw). */
tl_status tl_model_segment_time(double n_tokens, double d_q, double d_kv, double flops, double mem_bw,
                                double* seconds_out);
/* Section 4.1: T_comm = 2 * net_latency + 4 d_q / net_bw (query row out, partial row back). */
tl_status tl_model_comm_time(double d_q, double net_latency, double net_bw, double* seconds_out);
/* Section 4.1: the segment size (tokens, real-valued) from which T_comp >= T_comm. */
tl_status tl_model_segment_threshold(double d_q, double d_kv, double flops, double mem_bw, double net_latency,
                                     double net_bw, double* tokens_out);
/* Section 5.1 (get_cache_load): M_r = sum 4 d (prefix + input), F_r = sum 2 d prefix input,
 * L = max(M_r / (M_r + n_gpus mem_bw t_ideal), F_r / (F_r + n_gpus flops t_ideal)).
 * prefix_len / input_len: host [n].  Any of the three outputs may be NULL. */
tl_status tl_model_cache_load(double d, const int64_t* prefix_len, const int64_t* input_len, int32_t n,
                              int32_t n_gpus, double mem_bw, double flops, double t_ideal, double* traffic_out,
                              double* flops_out, double* load_out);

/* ------------------------------------------------------------------------------------
 * Segment ids from token content (Section 3.1: the global prefix tree is keyed by the token
 * sequence, so requests name the same cached segment exactly as far as their prompts agree).
 * Segment k of a sequence covers tokens [k seg_len, min(n_tokens, (k+1) seg_len)); its id is the
 * 64-bit FNV-1a hash of all tokens up to its end, each token as four little-endian bytes,
 * started from the offset basis xor `salt`.  Two sequences get equal ids for the whole segments
 * of their common prefix and (but for hash collisions) different ids from there on; a partly
 * filled last segment has an id of its own.  tokens: host [n_tokens]; ids_out: host
 * [ceil(n_tokens / seg_len)].  Host arithmetic, bit-exact.  TL_EINVAL for seg_len <= 0,
 * negative n_tokens or a null array that is needed.
 * ------------------------------------------------------------------------------------ */
tl_status tl_segment_ids(const int32_t* tokens, int64_t n_tokens, int32_t seg_len, uint64_t salt, uint64_t* ids_out);

#ifdef __cplusplus
}
#endif
#endif /* TOKENLAKE_H_ */
