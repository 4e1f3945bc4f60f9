/*
 * valvekv — preemptible paged-KV decode attention and KV memory reclamation
 * for one AMD MI355X (gfx950).  C ABI.
 *
 * The problem is the one stated for online-offline colocation in the Valve
 * paper: an offline decode job fills the KV memory an online tenant leaves
 * idle; when the online tenant needs compute or memory back, the offline job
 * must stop within a sub-millisecond bound (Section 2.3, Challenge 1;
 * Section 4), and KV memory must be handed back promptly, below layer
 * granularity, without faults and without killing the offline job
 * (Section 2.3, Challenge 2; Section 5, "Sub-layer memory reclamation").
 *
 * The paper answers with a driver-level channel switch and by discarding the
 * reclaimed KV.  This library answers cooperatively:
 *   - decode attention of a layer is issued as slices of bounded KV bytes, so a
 *     yield lands at the next slice boundary and later resumes from a cursor;
 *   - a reclaimed block range is emptied by copying its live blocks to free
 *     blocks outside it and rewriting every block-table entry, so the offline
 *     job keeps its KV and never reads handed-over memory.
 *
 * Conventions
 *   - Every function returns an int status: VKV_OK (0), VKV_YIELDED (1) or a
 *     negative VKV_E_* code.  vkv_last_error() gives a message for the calling
 *     thread's last failure.  No exception crosses this boundary.
 *   - "device" pointers are HIP device memory owned by the caller; "host"
 *     pointers are ordinary host memory owned by the caller.  The library owns
 *     only the opaque vkv_pool object (host memory, small pinned staging
 *     buffers, two progress words in pinned host memory that slice launches
 *     report to, HIP events, one extra stream once kv_sched_set_overlap has
 *     been used).  It never allocates or frees device memory; the one
 *     exception, at the caller's request, is the kv_arena_* group, and
 *     paged_decode_attn_layer_static works in a fixed 16 MiB device array that
 *     is part of the library's image.
 *   - Streams are hipStream_t passed as void* (NULL = the default stream).
 *     Device work is enqueued on the given stream; unless stated otherwise a
 *     call returns without waiting for it.
 *   - A pool may be driven by two host threads at once: one "decode" thread
 *     (kv_attn_plan / bind / check, paged_decode_attn_slice, kv_attn_run_layer)
 *     and one "memory" thread (kv_pool_*, kv_reclaim_*); the two groups touch
 *     disjoint state.  Within a group, one thread at a time.
 *     kv_yield_request / kv_yield_clear / kv_yield_pending are safe from any
 *     thread at any time.
 *
 * Pool layout (bf16 elements, block-major so that a block-id range is an
 * address range):   pool[block][layer][K=0|V=1][kv_head][slot][d]
 * with block_tokens (= 16) slots per block.
 */
#ifndef VALVEKV_H
#define VALVEKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VKV_OK          0
#define VKV_YIELDED     1   /* kv_attn_run_layer stopped at a slice boundary on request */
#define VKV_E_INVAL    (-1) /* bad argument, misaligned or out-of-bounds range; nothing changed */
#define VKV_E_NOSPACE  (-2) /* not enough free blocks; nothing changed */
#define VKV_E_BUSY     (-3) /* range overlaps one that is already handed over; nothing changed */
#define VKV_E_HIP      (-4) /* a HIP call failed; the pool must be destroyed */
#define VKV_E_STATE    (-5) /* call sequence error (e.g. slice without a bound plan) or
                               inconsistent tables found by a checker */

typedef struct vkv_pool vkv_pool;

/* Geometry of the shared KV pool: equal-size handles of blocks_per_handle
 * blocks each (Section 3: a global pool of coarse handles with an
 * allocate-release interface; Algorithm 1 requires equal-size handles). */
typedef struct vkv_pool_config {
  int32_t  num_layers;
  int32_t  num_q_heads;
  int32_t  num_kv_heads;        /* divides num_q_heads; group size G = q/kv <= 16 */
  int32_t  head_dim;            /* 64 or 128 */
  int32_t  block_tokens;        /* 16 */
  int32_t  num_blocks;          /* NB; multiple of blocks_per_handle */
  int32_t  blocks_per_handle;   /* reclaimed ranges are multiples of this */
  int32_t  reserved;
  void*    base;                /* device, 16-byte aligned, caller-owned; may be NULL for a
                                   host-only pool that is never used for device work */
  uint64_t bytes;               /* >= num_blocks * block_bytes */
} vkv_pool_config;

const char* vkv_last_error(void);

/* ---- pool (host-only bookkeeping; no device work) ---------------------- */

/* Validates the geometry and creates a pool in which every block is free.
 * Errors: VKV_E_INVAL. */
int kv_pool_init(const vkv_pool_config* cfg, vkv_pool** out);
int kv_pool_destroy(vkv_pool* pool);

/* Allocate-release interface (Section 3).  kv_pool_alloc hands out the n lowest
 * free block ids outside handed-over ranges (VKV_E_NOSPACE if fewer exist);
 * kv_pool_adopt marks the given free ids live (to build a fragmented state);
 * kv_pool_free releases live ids.  A bad id gives VKV_E_INVAL and no change. */
int kv_pool_alloc(vkv_pool* pool, int32_t n, int32_t* ids_out_host);
int kv_pool_adopt(vkv_pool* pool, const int32_t* ids_host, int32_t n);
int kv_pool_free(vkv_pool* pool, const int32_t* ids_host, int32_t n);

/* The online tenant gives back handles it holds: [lo,hi), a multiple of
 * blocks_per_handle, must lie inside one handed-over range, which shrinks or
 * splits accordingly (the dynamic reservation of Section 5 releases one handle at
 * a time); the blocks become free pool blocks again.  VKV_E_INVAL otherwise;
 * VKV_E_STATE if an arena is attached and the handles are unmapped. */
int kv_pool_return_range(vkv_pool* pool, int32_t lo_block, int32_t hi_block);

/* State read-back: live_out_host[NB] gets 1 for live blocks; ranges_out_host
 * gets up to cap (lo,hi) pairs of handed-over ranges, *n_ranges their count.
 * Either output may be NULL. */
int kv_pool_state(vkv_pool* pool, uint8_t* live_out_host,
                  int32_t* ranges_out_host, int32_t cap, int32_t* n_ranges);

/* Checks a host copy of block tables against the pool: every entry is -1 or a
 * live block outside every handed-over range.  VKV_E_STATE on the first
 * violation (message names entry and block). */
int kv_pool_check_tables(vkv_pool* pool, const int32_t* tables_host, int64_t n_entries);

/* ---- decode attention -------------------------------------------------- */

typedef struct vkv_attn_plan_info {
  int32_t  n_items;             /* work items = (sequence, kv head, chunk of tokens) */
  int32_t  n_slices;            /* launches per layer */
  uint64_t workspace_bytes;     /* device workspace the caller must provide */
  uint64_t kv_bytes_per_layer;  /* K+V bytes one layer's attention reads */
  uint64_t max_slice_kv_bytes;  /* largest slice */
} vkv_attn_plan_info;

/* Host only.  Cuts the decode batch into work items of at most chunk_tokens
 * consecutive tokens of one kv head (order: sequence, chunk, kv head) and groups
 * consecutive items into slices reading at most slice_bytes of K+V (at least
 * one item each), so that a yield request is honoured within one slice
 * (Section 2.3, Challenge 1: bounded preemption latency).
 * ctx_len_host[s] >= 0 counts the tokens already in the cache, the newest
 * included; 0 = the sequence is not in the batch (a request that was evicted
 * and went back to the waiting state, Section 5): it gets no work and its
 * output rows are not written.  chunk_tokens: multiple of 32 in [32, 2048].
 * Replaces any earlier plan.  Errors: VKV_E_INVAL. */
int kv_attn_plan(vkv_pool* pool, const int32_t* ctx_len_host, int32_t num_seqs,
                 uint64_t slice_bytes, int32_t chunk_tokens, vkv_attn_plan_info* info_out);

/* Copies the current plan to host arrays: work_out_host[n_items][4] =
 * (sequence, kv_head, first_block_index, n_tokens); slice_start_out_host[n_slices+1]. */
int kv_attn_plan_read(vkv_pool* pool, int32_t* work_out_host, int32_t* slice_start_out_host);

/* Enqueues the upload of the current plan into `workspace` (device,
 * >= workspace_bytes, 256-byte aligned) on `stream` and zeroes its progress
 * counters.  The workspace also holds the per-item partial results and the
 * per-(sequence, kv head) progress counters of the layer in flight; it is the
 * resume state after a yield and must not be touched by the caller between
 * slices of a layer.  A layer that was started must be finished (all its
 * slices run) before another layer uses the workspace; to abandon a layer,
 * bind again.  Blocks the host only if an earlier upload from the same pool is
 * still in flight.  Errors: VKV_E_INVAL, VKV_E_STATE (no plan), VKV_E_HIP. */
int kv_attn_bind(vkv_pool* pool, void* workspace, uint64_t workspace_bytes, void* stream);

/* Enqueues one slice of one layer: for every work item of the slice, scores
 * q.k/sqrt(D) (or * softmax_scale if nonzero) of the G query heads of the
 * item's kv head against the item's tokens, running maximum, sum of
 * exponentials and exp-weighted sum of V rows.  The item that completes a
 * (sequence, kv head) pair merges the pair's chunks (log-sum-exp merge, in chunk
 * order) and writes out[seq][head][:], so `out` is complete once every slice of
 * the layer has run; slices of a layer may run in any order and any number of
 * launches apart.  Query head g uses kv head g / G.  Token t of a sequence lives
 * in block block_table[seq][t / 16], slot t % 16; slots past the sequence length
 * are never read.  bf16 inputs, fp32 accumulation.
 *   q_bf16       device [num_seqs][num_q_heads][head_dim] for this layer
 *   block_table  device int32 [>= num_seqs rows][max_blk], -1 padded
 *   out_f32      device fp32 [num_seqs][num_q_heads][head_dim], 16-byte aligned
 * The host checks layer, slice and max_blk against the plan (VKV_E_INVAL,
 * VKV_E_STATE); the kernel skips table entries outside [0, NB) and raises a flag
 * that kv_attn_check reports. */
int paged_decode_attn_slice(vkv_pool* pool, int32_t layer, int32_t slice,
                            const void* q_bf16, const int32_t* block_table, int32_t max_blk,
                            void* workspace, void* out_f32, float softmax_scale, void* stream);

/* Waits for `stream` and returns VKV_E_STATE if any slice since the last bind
 * met a block-table entry outside [0, NB); VKV_OK otherwise. */
int kv_attn_check(vkv_pool* pool, void* workspace, void* stream);

/* Slice scheduler.  Issues slices *cursor_slice .. n_slices-1 of `layer`,
 * keeping at most max_inflight (1..8) launches unfinished so that the
 * host stays close to the device; the count carries over from one call to the
 * next (use one stream per pool for these calls).  With max_inflight >= 2 and
 * all slices on one stream the launches report their start through pinned host
 * memory that the host polls, so kernels follow each other directly; otherwise
 * an event is recorded behind every launch.  Before each slice it tests
 * the yield flag; if set it stops issuing, waits until the launches already
 * enqueued have finished, stores the next slice in *cursor_slice and returns
 * VKV_YIELDED: offline compute is then off the GPU, at most max_inflight
 * launches after the request.  A later call with the same cursor continues
 * without recomputing anything (the paper's requirement that preempted work is
 * resumed, not repeated: Section 2.2 on duplicated iterations; Section 4.1).
 * On VKV_OK *cursor_slice = n_slices and every slice has been enqueued (not
 * waited for).
 * A layer of four slices or more is merged differently from what
 * paged_decode_attn_slice does on its own: its slices store their partial
 * results only, and one small launch behind the layer's last slice (enqueued
 * with it, so a yield lands before that slice or after the merge) merges every
 * split (sequence, kv head) in chunk order and clears the progress counters; the
 * bits are the same.  Slices of such a layer that were enqueued on their own
 * before this call takes over (cursor > 0) are fine; the other way round is not:
 * a layer that this call has begun must be finished by this call, because its
 * slices have not counted their chunks for paged_decode_attn_slice to go by. */
int kv_attn_run_layer(vkv_pool* pool, int32_t layer, int32_t* cursor_slice,
                      const void* q_bf16, const int32_t* block_table, int32_t max_blk,
                      void* workspace, void* out_f32, float softmax_scale,
                      int32_t max_inflight, void* stream);

/* For callers that cannot allocate or be handed a workspace: code that is being
 * recorded into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.
 * One whole layer of decode attention as paged_decode_attn_slice computes it, in
 * one launch, with no plan, no bind and no workspace argument: the progress
 * counters and the per-chunk partial results live in a 16 MiB array that is part
 * of the library's device image (each GPU the library runs on holds its own copy
 * until the process ends).  The call allocates nothing and frees nothing, on the
 * device or through the runtime; it enqueues one small fill kernel (the counters
 * must start at zero whatever an earlier call left behind) and the attention
 * kernel on `stream`, and returns.
 *   ctx_len_dev    device int32 [num_seqs], every value in [1, max_ctx_tokens]
 *   max_ctx_tokens upper bound of the context lengths, <= max_blk * 16; the grid
 *                  has one workgroup per (sequence, chunk slot, kv head), and
 *                  workgroups past the end of their sequence exit at once
 *   chunk_tokens   as for kv_attn_plan; for equal chunk_tokens the output bits
 *                  equal those of the planned path
 *   err_flag_dev   device uint32, may be NULL: bit 0 is set if a block-table
 *                  entry outside [0, NB) was met (it is skipped), bit 1 if a
 *                  context length was outside [1, max_ctx_tokens] (it is clamped;
 *                  a sequence of length < 1 gets no output).  The caller clears it.
 *   other arguments as for paged_decode_attn_slice.
 * Limit: num_seqs * ceil(max_ctx_tokens / chunk_tokens) * kv_heads work items
 * whose counters and partial results fit the 16 MiB (VKV_E_NOSPACE otherwise, and
 * nothing is enqueued; the message gives the size needed).
 * All calls on one GPU share that GPU's array: two calls whose kernels may run
 * at the same time on one GPU (different streams, different threads) race;
 * calls on one stream, or otherwise ordered, are fine.  The first call on a
 * device looks the array's address up (no allocation); make that call outside
 * graph capture.  kv_pool_init does the lookup already when given device memory.
 * Errors: VKV_E_INVAL, VKV_E_NOSPACE, VKV_E_HIP. */
int paged_decode_attn_layer_static(vkv_pool* pool, int32_t layer, const void* q_bf16,
                                   const int32_t* block_table, int32_t max_blk,
                                   const int32_t* ctx_len_dev, int32_t num_seqs, int32_t max_ctx_tokens,
                                   int32_t chunk_tokens, void* out_f32, uint32_t* err_flag_dev,
                                   float softmax_scale, void* stream);

/* With enable != 0 the slice schedulers (kv_attn_run_layer, kv_prefill_run_layer)
 * send every other slice of a layer to a second stream owned by the pool
 * (created on first use, default priority), forked from and joined back into the
 * caller's stream inside the same call: the head of one launch fills the
 * compute units that the tail of the previous one leaves idle.  Ordering seen
 * by the caller is unchanged (work enqueued on `stream` before the call
 * precedes every slice; work enqueued after it follows every slice), results
 * are bit-identical, and at most max_inflight launches are unfinished as
 * before; it takes effect when max_inflight >= 2.  Off by default.  The first
 * enabling call creates the stream (the device of the pool must be current);
 * make it before a second thread starts using the pool: kv_reclaim_range's
 * grace wait covers this stream too and reads its handle.
 * Errors: VKV_E_INVAL, VKV_E_HIP. */
int kv_sched_set_overlap(vkv_pool* pool, int32_t enable);

/* Yield flag (the online tenant's "busy" edge of Section 4.2).  Thread-safe. */
int kv_yield_request(vkv_pool* pool);
int kv_yield_clear(vkv_pool* pool);
int kv_yield_pending(vkv_pool* pool);   /* 1 if set, 0 if not */

/* ---- reclamation ------------------------------------------------------- */

typedef struct vkv_reclaim_stats {
  uint64_t bytes_moved;         /* live bytes copied (read side) */
  int32_t  blocks_moved;
  int32_t  blocks_in_range;     /* hi - lo */
  int32_t  n_chunks;            /* copy launches */
  int32_t  reserved;
  double   host_seconds;        /* wall time of the call */
} vkv_reclaim_stats;

/* Host only, changes nothing.  Plans the relocation of range [lo,hi): the i-th
 * live block of the range (ascending) goes to the i-th free block (ascending)
 * outside the range and outside every handed-over range.  remap_out_host[NB]
 * (may be NULL) gets the identity except remap[src_i] = dst_i.
 * Errors: VKV_E_INVAL (range empty, out of bounds or not handle-aligned),
 * VKV_E_BUSY, VKV_E_NOSPACE. */
int kv_reclaim_plan(vkv_pool* pool, int32_t lo_block, int32_t hi_block,
                    int32_t* remap_out_host, vkv_reclaim_stats* stats_out);

#define VKV_RECLAIM_ASYNC 1u  /* return after enqueueing; the caller waits for copy_stream
                                 and guarantees that no slice is in flight */
#define VKV_RECLAIM_NO_GRACE 2u /* the caller guarantees that no slice of this pool is in flight
                                 on any stream: step 4 waits for copy_stream only */

/* Hands block range [lo,hi) to the online tenant (Section 5: stop offline
 * compute first, pick handles, make them harmless, hand them over):
 *   1. plan as kv_reclaim_plan; on error nothing has changed;
 *   2. copy live blocks out of the range on copy_stream, in launches of at most
 *      chunk_bytes of live data (0 = one launch); with rate_cap_bytes_per_s > 0
 *      launch j is not issued before t0 + (live bytes of launches < j) / cap
 *      (the host thread sleeps; burst allowance = one chunk);
 *   3. rewrite block_tables (device int32, n_entries entries, -1 = empty) in
 *      place: entry e becomes remap[e];
 *   4. wait for copy_stream; then, unless decode_stream is the same stream as
 *      copy_stream (stream order has done it already), wait until the work enqueued
 *      on decode_stream so far has finished: slices launched before the rewrite may
 *      have read old entries, which still point at intact source blocks.  NULL
 *      names the default stream here as everywhere.  The second stream of
 *      kv_sched_set_overlap, if there is one, is waited for in the same way;
 *   5. mark the range handed over.  From here no table entry and no later
 *      slice refers to it.
 * remap_dev: device int32 [NB] scratch, filled with the remap of this call.
 * With VKV_RECLAIM_ASYNC step 4 is skipped; with VKV_RECLAIM_NO_GRACE only its
 * first part is done.
 * Concurrent slices on decode_stream stay correct throughout: copies only write
 * free blocks, and both old and new table entries name identical bytes.
 * Errors: as kv_reclaim_plan, VKV_E_HIP. */
int kv_reclaim_range(vkv_pool* pool, int32_t lo_block, int32_t hi_block,
                     int32_t* block_tables, int64_t n_entries,
                     uint64_t chunk_bytes, uint64_t rate_cap_bytes_per_s,
                     void* copy_stream, void* decode_stream,
                     int32_t* remap_dev, uint32_t flags, vkv_reclaim_stats* stats_out);

/* Enqueues tables[i] = remap[tables[i]] for every entry in [0, num_blocks);
 * other entries (-1 padding) are left alone.  Exported on its own for tables the
 * pool does not know about (Section 5: the framework is told which block ids
 * changed). */
int block_table_rewrite(int32_t* tables_dev, int64_t n_entries, const int32_t* remap_dev,
                        int32_t num_blocks, void* stream);

/* ---- prefill attention (head_dim 128) ------------------------------------------- */

typedef struct vkv_prefill_plan_info {
  int32_t  n_items, n_slices, n_tiles;
  int32_t  tile_positions;      /* query positions per tile = 128 / (G rounded up to a power of two) */
  int32_t  total_q;             /* sum of q_len: rows of q and out */
  int32_t  n_merge_steps;       /* launches the merge of split tiles is cut into (>= 1) */
  uint64_t workspace_bytes;
  uint64_t kv_bytes_per_layer;  /* K+V bytes all items read (tokens are re-read once per query tile) */
  uint64_t max_slice_kv_bytes;
  double   flops_per_layer;     /* 4 * D * Hq * sum over queries of (position + 1): the causal attention itself */
} vkv_prefill_plan_info;

/* Host only.  Plans the causal attention of the newest q_len_host[s] tokens of
 * every sequence (positions ctx_len[s] - q_len[s] .. ctx_len[s] - 1; their K/V is
 * already in the cache) as preemptible slices: long prefills are where the
 * paper finds coarse preemption costliest (Section 2.2, Section 5).
 *   - the new tokens of a sequence are cut into tiles of tile_positions positions;
 *   - the tokens a tile can see (0 .. its last position) are cut into chunks of
 *     chunk_tokens (multiple of 32 in [32, 16384]);
 *   - work item = (tile, kv head, chunk), order tile, chunk, kv head;
 *   - a slice is a maximal run of items reading at most slice_bytes of K+V.
 * Query rows are packed: sequence s owns rows sum(q_len[:s]) .. + q_len[s].
 * Errors: VKV_E_INVAL (needs 1 <= q_len <= ctx_len; a pool whose head_dim is
 * not 128 is refused here, before any workspace is sized). */
int kv_prefill_plan(vkv_pool* pool, const int32_t* ctx_len_host, const int32_t* q_len_host, int32_t num_seqs,
                    uint64_t slice_bytes, int32_t chunk_tokens, vkv_prefill_plan_info* info_out);

/* work_out_host[n_items][4] = (tile, kv_head, first_block_index, n_tokens);
 * slice_start_out_host[n_slices+1]; tiles_out_host[n_tiles][4] = (sequence, first q
 * row, first position, positions); tile_base_out_host[n_tiles+1].  Any may be NULL. */
int kv_prefill_plan_read(vkv_pool* pool, int32_t* work_out_host, int32_t* slice_start_out_host,
                         int32_t* tiles_out_host, int32_t* tile_base_out_host);

/* As kv_attn_bind, for the prefill plan (its own workspace). */
int kv_prefill_bind(vkv_pool* pool, void* workspace, uint64_t workspace_bytes, void* stream);

/* Enqueues one slice: for every work item, causal scores q.k/sqrt(D) (or
 * * softmax_scale) of the tile's (position, query head) columns against the
 * item's tokens, running max / sum / weighted V sum per column; a token at
 * position t is visible to the query at position p iff t <= p.  Items that cover
 * everything their tile can see write out directly; the others leave partial
 * results in the workspace for kv_prefill_merge.
 *   q_bf16   device [total_q][num_q_heads][128]
 *   out_f32  device fp32 [total_q][num_q_heads][128], 16-byte aligned */
int paged_prefill_attn_slice(vkv_pool* pool, int32_t layer, int32_t slice,
                             const void* q_bf16, const int32_t* block_table, int32_t max_blk,
                             void* workspace, void* out_f32, float softmax_scale, void* stream);

/* Enqueues step `step` (0 .. n_merge_steps-1) of the merge of split tiles
 * (log-sum-exp, chunk order) into out; every slice of the layer must have been
 * enqueued on the same stream before.  The merge is cut into steps of bounded
 * size (partial results + outputs of at most slice_bytes / 2) so that it cannot
 * delay a yield by more than a slice does.  Steps are independent and idempotent. */
int kv_prefill_merge(vkv_pool* pool, int32_t step, void* workspace, void* out_f32, void* stream);

/* Slice scheduler for prefill: as kv_attn_run_layer, with the merge steps
 * following the slices: *cursor_slice runs over 0 .. n_slices + n_merge_steps
 * (that value on VKV_OK); a yield may land before any slice or merge step. */
int kv_prefill_run_layer(vkv_pool* pool, int32_t layer, int32_t* cursor_slice,
                         const void* q_bf16, const int32_t* block_table, int32_t max_blk,
                         void* workspace, void* out_f32, float softmax_scale,
                         int32_t max_inflight, void* stream);

/* As kv_attn_check. */
int kv_prefill_check(vkv_pool* pool, void* workspace, void* stream);

/* ---- policies (host only) ---------------------------------------------------- */

/* Selective handle reclamation (Algorithm 1, Section 5).  Handle h is blocks
 * [h*blocks_per_handle, (h+1)*blocks_per_handle).  Reqs(h) = rows of
 * tables_host (int32 [n_rows][max_blk], -1 = empty) with an entry in h;
 * Cost(r) = cost_host[r] (the tokens request r would have to recompute).
 * k times, among handles not yet handed over and not yet chosen, picks the one
 * whose not-yet-evicted requests cost least in total (ties: lowest handle),
 * then counts those requests as evicted.  handles_out[k] in pick order;
 * evicted_rows_out (room for n_rows, ascending) and the counts may be NULL.
 * Changes nothing in the pool.  Errors: VKV_E_INVAL, VKV_E_NOSPACE (k too large). */
int kv_select_handles(vkv_pool* pool, const int32_t* tables_host, int32_t n_rows, int32_t max_blk,
                      const int64_t* cost_host, int32_t k, int32_t* handles_out,
                      int32_t* evicted_rows_out, int32_t* n_evicted_out, int64_t* total_cost_out);

/* What evicting a given set of handles would cost: evicted_rows_out (room for
 * n_rows, ascending; may be NULL) = rows with an entry in one of the handles,
 * *total_cost_out = sum of their cost.  For comparing policies, e.g. the
 * first-in-first-out baseline of Section 7.2 (the first k handles not yet handed
 * over).  Changes nothing.  Errors: VKV_E_INVAL. */
int kv_handles_cost(vkv_pool* pool, const int32_t* tables_host, int32_t n_rows, int32_t max_blk,
                    const int64_t* cost_host, const int32_t* handles_host, int32_t k,
                    int32_t* evicted_rows_out, int32_t* n_evicted_out, int64_t* total_cost_out);

/* Hands the given handles to the online tenant WITHOUT saving their contents
 * (the paper's way, Section 5): their blocks stop being live, each handle becomes
 * a handed-over range [h*bph, (h+1)*bph), and every table entry that named one of
 * their blocks is reported as (row, column, block id) in row-major order: the
 * invalidated ids the framework needs to requeue the affected requests
 * (their remaining blocks are the framework's to free).  If more than `cap`
 * entries are affected, *n_inv_out gets the number needed, VKV_E_NOSPACE is
 * returned and nothing changes.
 * tables_dev (device copy of the same tables, may be NULL): when given, the
 * affected entries become -1 there too (an entry the kernels skip and flag), on
 * `stream`, using remap_dev (device int32 [NB]) as scratch, and the call waits for
 * `stream` and, as kv_reclaim_range does, for the slices already enqueued on
 * decode_stream: from then on nothing reads the handles, and they may be
 * unmapped (kv_arena_release).  Without tables_dev the library cannot know what
 * the device tables say, and kv_arena_release refuses these ranges.
 * Errors: VKV_E_INVAL, VKV_E_BUSY, VKV_E_NOSPACE, VKV_E_HIP. */
int kv_invalidate_handles(vkv_pool* pool, const int32_t* handles_host, int32_t k,
                          const int32_t* tables_host, int32_t n_rows, int32_t max_blk,
                          int32_t* inv_row_out, int32_t* inv_col_out, int32_t* inv_block_out,
                          int32_t cap, int32_t* n_inv_out,
                          int32_t* tables_dev, int32_t* remap_dev, void* stream, void* decode_stream);

typedef struct vkv_evict_info {
  int32_t mode;                 /* 0: the range was emptied by relocation; 1: handles were evicted */
  int32_t n_handles;            /* handles handed over by eviction */
  int32_t n_evicted;            /* requests (table rows) evicted */
  int32_t n_invalidated;        /* table entries that named a block of an evicted handle */
  int64_t total_cost;           /* sum of Cost(r) over the evicted requests */
} vkv_evict_info;

/* Eviction as one call (Section 5, "Sub-layer memory reclamation" and "Selective
 * handle reclamation"): k handles are chosen by Algorithm 1 as in
 * kv_select_handles and handed over without saving their contents; every request
 * (row) with a block in one of them is evicted whole: its row is cleared in
 * tables_host (updated in place) and, when given, in tables_dev (on `stream`, with
 * scratch_dev, device int32 [>= n_rows], as scratch; then `stream` and the slices
 * already enqueued on decode_stream are waited for); its blocks outside the chosen
 * handles are freed unless a surviving row still names them; every block of a
 * chosen handle dies.  handles_out[k] in pick order; evicted_rows_out (room for
 * n_rows, ascending, may be NULL); the invalidated entries as for
 * kv_invalidate_handles (lists may be NULL; more than `cap` of them: VKV_E_NOSPACE,
 * info->n_invalidated says how many, nothing changes).  The evicted requests are
 * the framework's to requeue; plan the next decode step with their context length
 * set to 0.  Errors: VKV_E_INVAL, VKV_E_NOSPACE (also: fewer than k handles left),
 * VKV_E_HIP. */
int kv_evict_handles(vkv_pool* pool, int32_t k, int32_t* tables_host, int32_t n_rows, int32_t max_blk,
                     const int64_t* cost_host, int32_t* tables_dev, int32_t* scratch_dev,
                     void* stream, void* decode_stream,
                     int32_t* handles_out, int32_t* evicted_rows_out,
                     int32_t* inv_row_out, int32_t* inv_col_out, int32_t* inv_block_out, int32_t cap,
                     vkv_evict_info* info_out);

/* Hands (hi - lo) / blocks_per_handle handles to the online tenant: by emptying
 * [lo,hi) as kv_reclaim_range does when the free blocks elsewhere suffice (then
 * tables_host follows the rewrite of tables_dev), otherwise, instead of failing
 * with VKV_E_NOSPACE, by kv_evict_handles of that many handles (not necessarily
 * those of [lo,hi): the ones that cost least).  info_out->mode says which.
 * Arguments as for the two calls; remap_dev doubles as the eviction's scratch. */
int kv_reclaim_or_evict(vkv_pool* pool, int32_t lo_block, int32_t hi_block,
                        int32_t* tables_dev, int32_t* tables_host, int32_t n_rows, int32_t max_blk,
                        const int64_t* cost_host, uint64_t chunk_bytes, uint64_t rate_cap_bytes_per_s,
                        void* copy_stream, void* decode_stream, int32_t* remap_dev, uint32_t flags,
                        int32_t* handles_out, int32_t* evicted_rows_out,
                        int32_t* inv_row_out, int32_t* inv_col_out, int32_t* inv_block_out, int32_t cap,
                        vkv_evict_info* info_out, vkv_reclaim_stats* stats_out);

/* Dynamic reservation (Section 5, "Dynamic MIAD-style memory reservation"): the
 * online tenant's headroom H, in handles.  The paper fixes only the 90 %
 * threshold; every other constant is a parameter. */
typedef struct vkv_miad_config {
  int32_t h_init, h_min, h_max; /* headroom bounds, handles */
  int32_t reserved;
  double  alpha;                /* > 1: H <- ceil(H * alpha) on a pressure event (at least +1) */
  double  pressure_frac;        /* pressure event when used >= pressure_frac * H; the paper: 0.9 */
  double  t_init, t_min, t_max; /* release interval T, seconds */
  double  t_up;                 /* > 1: T <- T * t_up while the event rate exceeds the target */
  double  t_down;               /* T <- T - t_down otherwise */
  double  window_s;             /* sliding window of the event rate */
  double  target_rate;          /* pressure events per second the user accepts */
} vkv_miad_config;
typedef struct vkv_miad vkv_miad;
typedef struct vkv_miad_step {
  int32_t headroom;             /* H after this observation */
  int32_t grow_by;              /* handles to reclaim from the offline tenant now */
  int32_t release;              /* 1: one handle goes back to the offline tenant */
  int32_t pressure_event;
  double  interval_s;           /* T after this observation */
} vkv_miad_step;
int kv_miad_init(const vkv_miad_config* cfg, vkv_miad** out);
int kv_miad_destroy(vkv_miad* m);
/* One observation: at time now_s (non-decreasing) the online tenant uses
 * used_handles of its headroom.  Pressure: H grows, the event enters the window,
 * T adapts.  Otherwise, once T has passed since the last release tick or
 * event: H shrinks by one if it stays above h_min and above the usage, T adapts. */
int kv_miad_observe(vkv_miad* m, double now_s, int32_t used_handles, vkv_miad_step* out);

/* Wake-up gate (Section 4.2): offline work is preempted the moment the online
 * tenant turns busy and may run again only after the online tenant has been idle
 * for T_cool = 2 G without interruption; G is the largest idle gap seen between
 * two busy periods of the same request (gaps between decode iterations),
 * starting from initial_gap_s. */
typedef struct vkv_gate vkv_gate;
int kv_gate_init(double initial_gap_s, vkv_gate** out);
int kv_gate_destroy(vkv_gate* g);
int kv_gate_online_busy(vkv_gate* g, double now_s, int64_t request_id); /* 1: preempt offline now; 0: already off */
int kv_gate_online_idle(vkv_gate* g, double now_s);
int kv_gate_poll(vkv_gate* g, double now_s);                            /* 1: offline may run */
int kv_gate_stats(vkv_gate* g, double* max_gap_s_out, int64_t* preemptions_out);

/* ---- per-launch timing ---------------------------------------------------- */

#define VKV_PROF_SLICE    0   /* paged_decode_attn_slice kernel; index = slice */
#define VKV_PROF_RELOCATE 1   /* all block copy launches of one kv_reclaim_range call;
                                 index = number of launches */
#define VKV_PROF_REWRITE  2   /* table rewrite kernel */
#define VKV_PROF_PREFILL  3   /* paged_prefill_attn_slice kernel; index = slice */
#define VKV_PROF_PREFILL_MERGE 4

typedef struct vkv_profile_record {
  int32_t kind;
  int32_t index;
  float   ms;                 /* device time of the launch (slice kernels: the dispatch's own start to end;
                                 copy and rewrite: between events recorded around the launches) */
} vkv_profile_record;

/* With max_records > 0 every kernel launch of this pool is timed with two
 * events until max_records launches have been recorded; 0 turns recording off
 * and frees the events.  Used for roofline measurement.  A slice launch
 * (decode or prefill) carries its two events itself (hipExtLaunchKernelGGL):
 * they take the dispatch's start and end, nothing is enqueued between the
 * kernel and its neighbours, and the figure is the kernel's duration as a
 * profiler reports it.  Copy and rewrite launches are bracketed by events
 * recorded on their stream, which adds a few microseconds to the figure. */
int kv_profile_enable(vkv_pool* pool, int32_t max_records);

/* Times only every stride-th slice launch (default 1 = every launch; copy and
 * rewrite launches are always timed), which keeps a timed run as close to an
 * untimed one as possible.  Errors: VKV_E_INVAL. */
int kv_profile_sample(vkv_pool* pool, int32_t stride);

/* Waits for the recorded launches to finish, writes up to cap records (launch
 * order) to out_host, their count to *n_out, and restarts recording at zero. */
int kv_profile_read(vkv_pool* pool, vkv_profile_record* out_host, int32_t cap, int32_t* n_out);

/* ---- handle-backed pool memory (optional) ------------------------------------
 * The paper allocates and releases KV memory in equal-size handles and a
 * reclaimed handle leaves the offline job for good (Section 5).  An arena is
 * one reservation of device address space of num_handles * handle_bytes with
 * one physical allocation per handle (HIP virtual-memory API).  Used as the
 * pool's memory, it lets a range that kv_reclaim_range has handed over be
 * unmapped, which returns its physical memory to the driver: any other
 * allocation on the device, another process's included, can then have it.
 * Giving the range back maps fresh memory at the same addresses, so block ids
 * and tables stay as they are.  These are the only calls that allocate device
 * memory, and only at the caller's request.  Memory thread. */
typedef struct vkv_arena vkv_arena;

/* Reserves the address range on `device` and backs every handle.  *base_out is
 * the device address to use as vkv_pool_config.base (bytes = num_handles *
 * handle_bytes; handle_bytes = blocks_per_handle * block bytes, a multiple of
 * the allocation granularity, 4 KiB here).
 * Errors: VKV_E_INVAL, VKV_E_NOSPACE (device memory), VKV_E_HIP. */
int kv_arena_create(int32_t device, uint64_t handle_bytes, int32_t num_handles, vkv_arena** arena_out,
                    void** base_out);
/* Unmaps what is mapped and frees the reservation.  Destroy the pool first. */
int kv_arena_destroy(vkv_arena* arena);

/* Tells the pool that its memory is this arena (NULL detaches).  Checks base,
 * handle size and total size.  With an arena attached, kv_pool_return_range
 * refuses (VKV_E_STATE) a range whose handles are unmapped. */
int kv_pool_attach_arena(vkv_pool* pool, vkv_arena* arena);

/* Unmaps the handles of [lo_block, hi_block) and releases their physical
 * memory.  The range (a multiple of blocks_per_handle) must lie inside one that
 * kv_reclaim_range, kv_evict_handles or kv_invalidate_handles has handed over
 * WITH the device block tables in hand and that has not been returned: by then
 * the copy or the clearing, the table rewrite and the grace wait are over, and
 * the allocator, the planner and every block table the library was shown avoid
 * it.  Any later access to it is a GPU fault.  Errors: VKV_E_INVAL (arena not
 * attached to this pool, bad range), VKV_E_STATE (not handed over, handed over
 * without the device tables, or already unmapped), VKV_E_HIP. */
int kv_arena_release(vkv_arena* arena, vkv_pool* pool, int32_t lo_block, int32_t hi_block);

/* Maps fresh physical memory (contents undefined) behind the handles of a
 * handed-over, unmapped range; follow with kv_pool_return_range.  On failure
 * the whole range stays unmapped.  Errors: VKV_E_INVAL, VKV_E_STATE,
 * VKV_E_NOSPACE (the device has no memory left), VKV_E_HIP. */
int kv_arena_restore(vkv_arena* arena, vkv_pool* pool, int32_t lo_block, int32_t hi_block);

/* mapped_out_host[num_handles] (1 = backed by physical memory), may be NULL;
 * *mapped_bytes_out = bytes currently backed, may be NULL. */
int kv_arena_state(vkv_arena* arena, uint8_t* mapped_out_host, uint64_t* mapped_bytes_out);

/* ---- bandwidth yardsticks ---------------------------------------------------
 * Not part of the method: the attention and relocation kernels are bound by
 * HBM bandwidth, and these two calls measure what the memory system gives the
 * simplest patterns on the same device, so a kernel can be quoted against the
 * reachable rate as well as against the data-sheet peak.  The caller times
 * them (events on `stream`). */

/* Launches a read-only kernel that streams src_dev[0, bytes) once,
 * sequentially, 64 KiB per workgroup.  sink_dev: 256 bytes of device scratch
 * (written only if the xor of the data equals one fixed 128-bit value).
 * bytes: positive multiple of 16; both pointers 16-byte aligned.
 * Errors: VKV_E_INVAL, VKV_E_HIP. */
int kv_probe_read(const void* src_dev, uint64_t bytes, void* sink_dev, void* stream);

/* Launches, for one slice of the bound plan, a kernel that performs the memory
 * reads of paged_decode_attn_slice (same work items, same 4 KiB runs of K and V,
 * same number of requests in flight) and none of its arithmetic: the rate this
 * reaches is what the access pattern allows.  Arguments as for
 * paged_decode_attn_slice; sink_dev: 256 bytes of device scratch, 16-byte aligned.
 * Errors: as paged_decode_attn_slice. */
int kv_probe_attn_reads(vkv_pool* pool, int32_t layer, int32_t slice, const int32_t* block_table,
                        int32_t max_blk, void* workspace, void* sink_dev, void* stream);

/* Enqueues the runtime's own device-to-device copy of bytes bytes (regions must
 * not overlap).  Errors: VKV_E_INVAL, VKV_E_HIP. */
int kv_probe_copy(void* dst_dev, const void* src_dev, uint64_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VALVEKV_H */
