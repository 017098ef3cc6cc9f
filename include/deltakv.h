/*
 * deltakv -- delta-prefill attention over a pooled, prefix-aliased KV cache (MI355X / gfx950).
 *
 * C ABI of the library.  Plain C types only.  Every pointer argument is marked
 * HOST or DEVICE.  Device buffers and the pinned host staging memory are allocated
 * and owned by the caller; the library owns host metadata only.
 *
 * General rules
 *   - every function returns an int32_t status (DK_OK == 0, errors negative), never
 *     throws, aborts or prints;
 *   - a call that fails leaves the pool's state unchanged;
 *   - calls that launch GPU work (dk_kv_append, dk_delta_attend, dk_append_attend,
 *     dk_delta_attend_noalloc, dk_seq_gather, dk_verify_greedy) are
 *     asynchronous on the HIP stream passed as `stream` (a hipStream_t cast to void*,
 *     NULL = the default stream).  They never wait for the device and never allocate
 *     device or pinned memory: descriptors travel through the caller's staging memory
 *     (dk_pool_desc::host_staging), and a call that finds every staging buffer still
 *     in flight returns DK_ERR_BUSY instead of waiting (dk_staging_wait is the matching wait).
 *     They read the slot metadata
 *     at call time, so later host-side calls (trim, release, alias) do not affect
 *     work already enqueued.  All GPU-launching calls on one pool must be issued on
 *     one stream, or be ordered by the caller;
 *   - host-only calls are thread-safe (one mutex per pool, paper Sec. 3.1).
 *
 * Vocabulary (paper Sec. 2.2, 3.1, 3.3): a *slot* is one named sequence sigma_i of the
 * pool; a *cell* holds one token's K and V for all KV heads; n is the number of tokens a
 * slot already caches, Delta the number of new tokens of this call.
 */
#ifndef DELTAKV_H
#define DELTAKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dk_pool dk_pool; /* opaque */

enum { DK_F32 = 0, DK_BF16 = 1 };

enum {
  DK_OK = 0,
  DK_ERR_INVALID = -1,     /* bad argument or a state the call does not allow */
  DK_ERR_TIMEOUT = -2,     /* dk_seq_acquire: no free slot within the timeout */
  DK_ERR_NO_CELLS = -3,    /* the arena cannot hold the cells an append needs */
  DK_ERR_NO_SLOT = -4,     /* slot id out of range or not acquired */
  DK_ERR_DUP_SLOT = -5,    /* the same slot listed twice in one batched call */
  DK_ERR_UNSUPPORTED = -6, /* shape / dtype / alias form the library does not implement */
  DK_ERR_WORKSPACE = -7,   /* workspace missing or too small */
  DK_ERR_HIP = -8,         /* a HIP runtime call failed (see dk_last_hip_error) */
  DK_ERR_BUSY = -9,        /* every staging buffer still carries an unfinished upload: nothing was enqueued;
                              synchronise the stream (or wait for earlier work) and call again */
  DK_ERR_NO_MEMORY = -10   /* the host ran out of memory for metadata */
};

/*
 * Pool description (paper Sec. 3.1: one unified inference context allocated once, whose
 * sequence-id space is a fixed pool split into a transient and a session region).
 *
 * Arena layout, DEVICE memory, caller-owned, must outlive the pool:
 *   k_arena[kv_head][cell][d], v_arena[kv_head][cell][d]   (head-major, d contiguous)
 *   each arena_cells * n_kv_heads * head_dim elements of `dtype`, 256-byte aligned.
 * Cells are handed out in granules of `granule_cells` consecutive cells (0 selects 256);
 * arena_cells is rounded down to whole granules.
 * Slot ids [0, n_slots - n_session_slots) form the transient region, the rest the
 * session region.
 * dev_meta: DEVICE scratch of at least dk_meta_bytes() bytes, caller-owned, used for
 * the per-call copy tables of dk_kv_append / dk_seq_gather.
 * host_staging: HOST memory, pinned (hipHostMalloc), 256-byte aligned, caller-owned, must outlive
 * the pool.  It is cut into staging_depth (0 selects 8, at most 64) equal buffers of at least
 * 64 KiB through which the descriptors of a launching call are uploaded; dk_staging_bytes() is the
 * recommended size (1 MiB per buffer).  A call whose descriptors exceed one buffer, or any call
 * that needs an upload on a pool created with host_staging == NULL, returns DK_ERR_WORKSPACE
 * (appends of at most 896 tokens need no upload).  NULL is meant for host-only use of the pool.
 */
typedef struct {
  int32_t n_slots;
  int32_t n_session_slots;
  int64_t arena_cells;
  int32_t granule_cells;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;
  int32_t dtype; /* DK_F32 or DK_BF16: element type of the arena, Q, K/V inputs and O */
  void* k_arena; /* DEVICE */
  void* v_arena; /* DEVICE */
  void* dev_meta; /* DEVICE */
  int64_t dev_meta_bytes;
  void* host_staging; /* HOST, pinned; NULL: no staging */
  int64_t host_staging_bytes;
  int32_t staging_depth;
} dk_pool_desc;

/* Bytes of dev_meta a pool of this description needs.  HOST only. */
int32_t dk_meta_bytes(const dk_pool_desc* desc, int64_t* bytes_out);
/* Recommended bytes of host_staging for this description (staging_depth buffers of 1 MiB).  HOST only. */
int32_t dk_staging_bytes(const dk_pool_desc* desc, int64_t* bytes_out);

/*
 * pool_create (paper Sec. 3.1).  Builds the slot table, the two free lists and the cell
 * allocator.  Touches no device memory and allocates none; with host_staging it creates one HIP
 * event per staging buffer (needs a current device).  DK_ERR_INVALID on a malformed description,
 * DK_ERR_UNSUPPORTED for head_dim not in {64, 128}, n_q_heads not a multiple of
 * n_kv_heads, or an unknown dtype.
 */
int32_t dk_pool_create(const dk_pool_desc* desc, dk_pool** pool_out);
int32_t dk_pool_destroy(dk_pool* pool);

/*
 * Slot lifecycle (paper Sec. 3.1: acquire from the region's free list, block with a
 * configurable timeout when it is empty, return the slot on completion).
 * region: 0 transient, 1 session.  timeout_ms < 0 waits without limit, 0 polls.
 * dk_seq_release empties the slot and returns it to its region's free list; cells that an
 * alias still references stay intact until the last reference goes (Sec. 3.3: a trie node
 * names the donor whose state still holds the matched cells).
 */
int32_t dk_seq_acquire(dk_pool* pool, int32_t region, int64_t timeout_ms, int32_t* slot_out);
int32_t dk_seq_release(dk_pool* pool, int32_t slot);
int32_t dk_seq_len(dk_pool* pool, int32_t slot, int64_t* len_out);

/*
 * seq_alias: SeqAlias(donor, dst, 0, m) of paper Alg. 1 / Sec. 3.3.  Metadata only: dst's
 * positions [0, p1) become the donor's cells; no K/V byte is read or written and the
 * cost does not depend on p1.  Requires p0 == 0 (else DK_ERR_UNSUPPORTED), donor != dst,
 * 0 <= p1 <= len(donor) and len(dst) == 0 (else DK_ERR_INVALID).  p1 == 0 is a no-op.
 * Afterwards donor and dst grow independently: each one's appends are invisible to the other.
 */
int32_t dk_seq_alias(dk_pool* pool, int32_t donor, int32_t dst, int64_t p0, int64_t p1);

/*
 * seq_trim: roll a slot back to new_len <= len tokens (paper Alg. 2, last step: drop the
 * rejected speculative tokens).  Metadata only.  Cells other slots still see are kept.
 */
int32_t dk_seq_trim(dk_pool* pool, int32_t slot, int64_t new_len);
/*
 * The same for a whole batch in one call (the trim after a batched verification step): slots HOST [n_seqs]
 * distinct, new_len HOST int64 [n_seqs].  All or nothing: DK_ERR_NO_SLOT / DK_ERR_DUP_SLOT / DK_ERR_INVALID
 * (a new_len above the slot's length) leave every slot as it was.
 */
int32_t dk_seq_trim_batch(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int64_t* new_len);

/*
 * kv_append: write new tokens' K and V into the slots' next cells (the cache write of
 * Decode(sigma, batch) in paper Alg. 1 / Alg. 2; only the delta cells are committed).
 *   slots     HOST  [n_seqs]     distinct acquired slot ids
 *   cu_delta  HOST  [n_seqs+1]   cu_delta[0] == 0, non-decreasing; entry b owns packed
 *                                token rows cu_delta[b] .. cu_delta[b+1]-1
 *   n_accept  HOST  [n_seqs] or NULL: append only the first n_accept[b] tokens of entry b
 *                                (speculative verify: 1 + accepted drafts)
 *   k_new, v_new  DEVICE [cu_delta[n_seqs], n_kv_heads, head_dim] token-major, contiguous
 * On success len(slot_b) grows by the appended count.  DK_ERR_NO_CELLS if the arena cannot
 * hold all of them (nothing is written, no length changes).
 */
int32_t dk_kv_append(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta,
                     const int32_t* n_accept, const void* k_new, const void* v_new, void* stream);

/*
 * kv_reserve: the bookkeeping half of dk_kv_append without the copy, for callers whose own kernels
 * write K/V straight into the arena (e.g. a fused projection epilogue).  Same arguments and errors
 * as dk_kv_append; cells_out HOST int64 [cu_delta[n_seqs]] receives the destination cell of every
 * token (-1 for tokens beyond n_accept).  HOST only, launches nothing.
 */
int32_t dk_kv_reserve(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta,
                      const int32_t* n_accept, int64_t* cells_out);

/*
 * delta_attend: for every entry b and each of its Delta_b new tokens i, causal softmax
 * attention of the token's query heads over the slot's n_b cached tokens plus new tokens
 * 0..i (absolute positions 0 .. n_b+i), query head h reading KV head h / (n_q_heads /
 * n_kv_heads).  Covers the batched variable-length delta prefill of paper Alg. 1 and the
 * Delta = k+1 verification batch of Alg. 2.
 *   q      DEVICE [cu_delta[n_seqs], n_q_heads, head_dim]
 *   k_new, v_new  both NULL: "appended" mode, the Delta_b new tokens are already the last
 *          Delta_b cells of slot b (n_b = len - Delta_b; Delta_b > len is DK_ERR_INVALID);
 *          both non-NULL (DEVICE, layout as in dk_kv_append): "staged" mode, n_b = len and
 *          the new tokens' K/V are read from these buffers, the cache is not modified.
 *   scale  multiplies the raw dot products before the softmax
 *   out    DEVICE [cu_delta[n_seqs], n_q_heads, head_dim], same dtype as q
 *   lse    DEVICE float [cu_delta[n_seqs], n_q_heads] or NULL: natural-log-sum-exp of the
 *          scaled scores of each row
 *   workspace  DEVICE, 256-byte aligned, at least dk_attend_workspace_bytes() for the same
 *          (slots, cu_delta, mode) and the same slot lengths; DK_ERR_WORKSPACE otherwise
 *          (dk_attend_workspace_bytes: staged = 0 appended mode, 1 staged mode, 2 dk_append_attend)
 * Entries with Delta_b == 0 produce no rows; n_b == 0 is legal.
 */
int32_t dk_attend_workspace_bytes(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta,
                                  int32_t staged, int64_t* bytes_out);
int32_t dk_delta_attend(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta, const void* q,
                        const void* k_new, const void* v_new, float scale, void* out, float* lse, void* workspace,
                        int64_t workspace_bytes, void* stream);

/*
 * append_attend: Decode(sigma, batch) of paper Alg. 1 as one call -- appends all Delta_b new tokens of every entry
 * to its slot and attends them (row i of entry b over the slot's n_b = len tokens before the call plus new tokens
 * 0..i).  The final pool state and the results are those of dk_kv_append (n_accept NULL) followed by
 * dk_delta_attend in appended mode; the K/V rows are written into the arena by the attention kernels themselves, so
 * no separate copy kernel runs.  A speculative step (Alg. 2) appends its k+1 rows this way and drops the rejected
 * ones afterwards with dk_seq_trim / dk_seq_trim_batch.
 *   k_new, v_new  DEVICE, required (layout as in dk_kv_append); the other arguments as in dk_delta_attend
 *   workspace     at least dk_attend_workspace_bytes(..., staged = 2, ...) for the same batch and slot lengths
 * Errors as for the two calls it replaces (DK_ERR_NO_CELLS: nothing appended, nothing launched); a failing call
 * leaves the lengths unchanged.
 */
int32_t dk_append_attend(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta, const void* q,
                         const void* k_new, const void* v_new, float scale, void* out, float* lse, void* workspace,
                         int64_t workspace_bytes, void* stream);

/*
 * delta_attend for callers that cannot allocate and have no workspace to hand over: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * dk_delta_attend without the workspace pair: the call's descriptors and split partials live in an array of
 * DK_STATIC_SCRATCH_BYTES that is part of the library's device image (every GPU the library runs on holds its
 * copy until the process ends).  The call allocates no device or pinned memory.  A batch that needs more than
 * DK_STATIC_SCRATCH_BYTES -- dk_attend_workspace_bytes() says how much it needs -- returns DK_ERR_WORKSPACE
 * and launches nothing: decode and verification batches need tens of KiB, prefill turns whose key range is
 * split need (splits x packed rows x KV heads x 520) bytes on top.
 * All calls on one GPU share that GPU's array, whatever pool they use: calls that may overlap on the device
 * (different streams without an ordering between them) race.  Nothing has to be cleared between calls: every
 * byte a call reads from the array it has written itself.
 */
#define DK_STATIC_SCRATCH_BYTES (32 << 20)
int32_t dk_delta_attend_noalloc(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta,
                                const void* q, const void* k_new, const void* v_new, float scale, void* out,
                                float* lse, void* stream);

/*
 * verify_greedy: the step after the Delta = k+1 verification pass of paper Alg. 2, on the device
 * (Sec. 3.8: greedy sampling is an argmax over the vocabulary logits, batched over the k+1
 * speculated positions, and the host never scans the logits).  Slot b's batch rows
 * cu_delta[b] .. cu_delta[b+1]-1 hold the tokens [G_last, draft 0, ..., draft k-1]; logits row s is
 * the model's output after batch position s.  For every row the kernel takes the argmax (ties: lowest
 * token id; a NaN logit counts as +infinity), then accepts drafts front to back while
 * argmax(row s) == draft s.  With `a` accepted drafts:
 *   n_keep[b]     = 1 + a   -- how many of the slot's k+1 new cells stay (the n_accept of dk_kv_append,
 *                              or len - (k+1) + n_keep as the new_len of dk_seq_trim)
 *   next_token[b] = argmax(row a), the token to emit next
 * Slots without rows get n_keep 0 and next_token -1.  Stateless: needs no pool.
 *   cu_delta_dev  DEVICE int32 [n_seqs+1]  (a device copy of the batch's cu_delta)
 *   logits        DEVICE [total_rows, row_stride] of dtype DK_F32 / DK_BF16, 16-byte aligned, row_stride
 *                 (elements, >= vocab) a multiple of 16 bytes; DK_ERR_UNSUPPORTED otherwise
 *   batch_tokens  DEVICE int32 [total_rows]
 *   argmax_out    DEVICE int32 [total_rows] or NULL
 *   n_keep_out, next_token_out  DEVICE int32 [n_seqs]
 *   workspace     DEVICE, 256-byte aligned, >= dk_verify_workspace_bytes(total_rows, vocab, dtype)
 * total_rows <= 65535, vocab < 2^31.  Asynchronous on `stream`; allocates nothing.
 */
int32_t dk_verify_workspace_bytes(int32_t total_rows, int64_t vocab, int32_t dtype, int64_t* bytes_out);
int32_t dk_verify_greedy(int32_t n_seqs, int32_t total_rows, const int32_t* cu_delta_dev, const void* logits,
                         int32_t dtype, int64_t vocab, int64_t row_stride, const int32_t* batch_tokens,
                         int32_t* argmax_out, int32_t* n_keep_out, int32_t* next_token_out, void* workspace,
                         int64_t workspace_bytes, void* stream);

/*
 * Radix prefix cache and the per-turn procedure of paper Alg. 1 (Sec. 3.3), HOST only.  The trie is keyed
 * by token ids; a node owns a token segment and names a donor sequence (a slot of the pool's session
 * region that aliases the saver's cells) holding the whole path down to it.
 *   dk_radix_create   cell_budget: most cells the trie may hold (sum of its nodes' segment lengths, the
 *                     "cell budget" of Sec. 3.2); keep_last: tokens that always go through the model even
 *                     when the whole prompt is cached (1: the turn needs logits for its last position).
 *                     Destroy the trie before its pool; destroying it releases the donor slots.
 *   dk_radix_begin_turn  Alg. 1 lines 1-5: (m, donor) = longest cached prefix of tokens[0..n_tokens), capped at
 *                     n_tokens - keep_last; if m > 0, SeqAlias(donor, slot, 0, m) -- so `slot` must be acquired
 *                     and empty (errors of dk_seq_alias are passed on).  *n_past_out = m, the cells skipped this
 *                     turn.  The caller then runs only tokens[m..] through dk_kv_append / dk_delta_attend.
 *   dk_radix_save     Alg. 1 last line, once len(slot) >= n_tokens: walk the branch to its tip (splitting a node
 *                     if the prompt diverges inside its segment) and append ONE node holding only the cells the
 *                     trie does not have yet.  If that would exceed the budget, or no session slot is free, the
 *                     leaf with the oldest touch is shed (never a node on this save's own path) until it fits;
 *                     *saved_out (nullable) = 1 if the prompt is now cached to its end, 0 if room could not be
 *                     made (not an error: the turn is unaffected).
 *   dk_radix_stats    nodes, cells held, donor slots held, leaves shed so far (each pointer nullable).
 *   dk_radix_evicted_path  token path (root to leaf end) of the index-th shed leaf, oldest first: *len_out =
 *                     its length, at most cap tokens copied; DK_ERR_INVALID if there is no such leaf.
 * Calls on one trie are serialised by a mutex of its own.
 */
typedef struct dk_radix dk_radix;
int32_t dk_radix_create(dk_pool* pool, int64_t cell_budget, int32_t keep_last, dk_radix** radix_out);
int32_t dk_radix_destroy(dk_radix* radix);
int32_t dk_radix_begin_turn(dk_radix* radix, int32_t slot, const int32_t* tokens, int64_t n_tokens,
                            int64_t* n_past_out);
int32_t dk_radix_save(dk_radix* radix, int32_t slot, const int32_t* tokens, int64_t n_tokens, int32_t* saved_out);
int32_t dk_radix_stats(dk_radix* radix, int64_t* nodes_out, int64_t* cells_out, int64_t* donors_out,
                       int64_t* evictions_out);
int32_t dk_radix_evicted_path(dk_radix* radix, int64_t index, int32_t* tokens_out, int64_t cap, int64_t* len_out);

/*
 * Prompt-lookup drafting, HOST only (paper Sec. 3.6, Alg. 2 line 1: LookupNgram(R, G_tail, l, N)).
 * dk_pld_lookup: `recent` is the slot's recent token buffer (prompt followed by its own output).  Finds the
 *   largest n in [min_match, max_match] such that the buffer's last n tokens also occur ending before its last
 *   token (the most recent such occurrence among equals) and copies the tokens that followed it, at most
 *   max_draft, to draft_out (HOST int32 [max_draft]).  *n_draft_out = k (0: no confident match),
 *   *match_len_out (nullable) = n.
 * dk_pld_gate: acceptance gating.  *ema_inout <- (1 - beta) ema + beta accepted / proposed (unchanged when
 *   proposed == 0); *next_len_out = max_len if the average is >= threshold, else floor_len.
 */
int32_t dk_pld_lookup(const int32_t* recent, int64_t n_recent, int32_t min_match, int32_t max_match,
                      int32_t max_draft, int32_t* draft_out, int32_t* n_draft_out, int32_t* match_len_out);
int32_t dk_pld_gate(float* ema_inout, int32_t proposed, int32_t accepted, float beta, float threshold,
                    int32_t floor_len, int32_t max_len, int32_t* next_len_out);

/*
 * Scheduler helpers, HOST only (paper Sec. 3.2).
 * dk_prefill_chunk: workload-adaptive chunked prefill, chunk = clamp(n_batch / n_prefilling, 128, 4096); the
 *   ceiling narrows to 1024 when a latency-sensitive request is co-resident under contention
 *   (latency_sensitive != 0 and n_prefilling > 1).
 * dk_fnv1a32: 32-bit FNV-1a of a byte string (the hash of Sec. 3.2's prefix grouping and of Eq. 7).
 * dk_prefill_groups: prefix-aware grouped prefill.  Slot i has prompt tokens[i][0..n_tokens[i]) of which
 *   n_past[i] are already cached through radix prefix prefix_id[i] (any id that is equal for equal cached
 *   prefixes, e.g. the donor slot).  Slots with the same prefix_id and n_past whose next `window` tokens are
 *   identical (found by FNV-1a of those tokens' bytes, confirmed by comparison) form a group: the first of
 *   them in batch order is the leader (leader_out[i] = its index, i itself for leaders and ungrouped slots)
 *   and shared_out[i] = length of the prefix follower i has in common with its leader (>= n_past[i] + window;
 *   n_past[i] for leaders): after the leader has prefilled that far the follower takes it over with
 *   dk_seq_alias(leader_slot, slot_i, 0, shared_out[i]) instead of a forward pass.  The paper's window is K = 8.
 */
int32_t dk_prefill_chunk(int64_t n_batch, int32_t n_prefilling, int32_t latency_sensitive, int64_t* chunk_out);
int32_t dk_fnv1a32(const void* bytes, int64_t n_bytes, uint32_t* hash_out);
int32_t dk_prefill_groups(int32_t n_slots, const int32_t* const* tokens, const int64_t* n_tokens,
                          const int64_t* n_past, const int32_t* prefix_id, int32_t window, int32_t* leader_out,
                          int64_t* shared_out);

/*
 * Probes used by the tests to check bookkeeping bit for bit.
 * dk_seq_cells: physical cell index of each logical position (HOST int64 [cap]); writes
 *   min(len, cap) entries.  Aliased positions report the donor's cells.
 * dk_seq_gather: copy the slot's logical contents out as DEVICE [len, n_kv_heads, head_dim].
 * dk_pool_stats: cells currently allocated to live sequences / chains, and free cells.
 * dk_seq_stats: how the slot's logical contents lie in the arena -- the number of runs of consecutive cells
 *   (each run boundary costs the attention kernels a partly filled key tile) and the number of alias
 *   generations behind the slot (what the constant-time alias walks).  Each pointer nullable.
 */
int32_t dk_seq_cells(dk_pool* pool, int32_t slot, int64_t* cells_out, int64_t cap);
int32_t dk_seq_gather(dk_pool* pool, int32_t slot, void* k_out, void* v_out, void* stream);
int32_t dk_pool_stats(dk_pool* pool, int64_t* cells_held_out, int64_t* cells_free_out);
int32_t dk_seq_stats(dk_pool* pool, int32_t slot, int64_t* segments_out, int64_t* chain_nodes_out);

/*
 * Back-pressure for a caller that got DK_ERR_BUSY: blocks the calling HOST thread until the staging buffer that the
 * next launching call would take is free again (the upload that last used it has run), and no longer -- work queued
 * behind that upload keeps the device busy meanwhile, unlike after a stream synchronisation.  The only call besides
 * dk_pool_destroy and dk_attend_times that waits.  DK_ERR_WORKSPACE for a pool without staging memory.
 */
int32_t dk_staging_wait(dk_pool* pool);

/* Kernel selection for dk_delta_attend: 0 automatic (default), 1 force the scalar reference kernel. */
int32_t dk_set_attend_variant(dk_pool* pool, int32_t variant);
/*
 * Planner tuning, per pool; the defaults suit an MI355X (256 compute units in 8 XCDs) and the library
 * reads no environment variable.  Names and ranges (DK_ERR_UNSUPPORTED for an unknown name,
 * DK_ERR_INVALID for a value out of range or not whole where a count is meant):
 *   stream_rows       most packed query rows (G * Delta) of a sequence that still    [32, 96]       default 96
 *                     goes to the streaming kernel (more: the tile kernel)
 *   stream_target     aimed number of streaming work items per KV head             [1, 2^20]      default 256 / Hkv
 *   stream_min_chunk  smallest key range worth its own streaming item               [64, 2^24]     default 512
 *   stream_chains     workgroups of the streaming kernel (one per compute unit)     [1, 65536]     default 256
 *   stream_item_cost  fixed cost of a streaming unit in the chain balance, in keys  [0, 2^20]      default 512
 *   stream_queue      1: with four or more units per streaming workgroup the units   {0, 1, 2}      default 1
 *                     are drawn from a queue at run time (longest first);
 *                     2: already with more units than workgroups;
 *                     0: the workgroups always walk chains balanced on the host
 *   tile_wave_slots   tile-kernel workgroups of one KV head that run at a time      [1, 65536]     default 256 / Hkv
 *   tile_min_chunk    smallest key range worth its own tile item                    [64, 2^24]     default 128
 *   tile_item_cost    fixed cost of a tile item inside a chain, in 64-key tiles     [0, 65536]     default 5
 *   xcd_speed0 .. xcd_speed7  relative K/V streaming rate of each XCD, used when    (0, 100]       default 1 (even),
 *                     streaming chains are balanced on the host                                      0.95 (odd)
 * Affects only how later calls cut and order their work, never their results' meaning.
 */
int32_t dk_set_tuning(dk_pool* pool, const char* name, double value);
/*
 * Device time of the attention work (tile, streaming and merge kernels; not the descriptor upload) of recent
 * dk_delta_attend calls on this pool, measured with HIP events recorded on the call's stream.
 * dk_set_attend_timing(pool, n): keep the last n calls (0 <= n <= 256; 0 switches recording off).
 * dk_attend_times: waits for the recorded work, then writes the durations in milliseconds, oldest
 * first, of the last min(cap, recorded) calls to ms_out (HOST float [cap]); *n_out receives the count.
 * dk_last_attend_ms: the most recent one; DK_ERR_INVALID if nothing was recorded.
 */
int32_t dk_set_attend_timing(dk_pool* pool, int32_t n_calls);
int32_t dk_attend_times(dk_pool* pool, float* ms_out, int32_t cap, int32_t* n_out);
int32_t dk_last_attend_ms(dk_pool* pool, float* ms_out);

/*
 * Host time the launching calls of this pool have spent, by phase, in microseconds since the last reset
 * (a profiling probe: a few clock reads per call).  us_out HOST double [DK_HOST_PHASES] indexed by the
 * enum below, calls_out HOST int64 [2]: number of dk_delta_attend(_noalloc) and of dk_kv_append calls.
 * Each pointer nullable; reset != 0 clears the sums.
 */
enum {
  DK_HOST_PLAN = 0,          /* delta_attend: argument checks, resolving slots to segments, cutting work items */
  DK_HOST_STAGE = 1,         /* delta_attend: descriptors copied into the staging buffer */
  DK_HOST_UPLOAD = 2,        /* delta_attend: hipMemcpyAsync of the descriptors + its event */
  DK_HOST_LAUNCH = 3,        /* delta_attend: kernel launches (and timing events when recording) */
  DK_HOST_APPEND_BOOK = 4,   /* kv_append: bookkeeping (cells reserved, lengths advanced) */
  DK_HOST_APPEND_LAUNCH = 5, /* kv_append: table upload if any, kernel launch */
  DK_HOST_PHASES = 6
};
int32_t dk_host_times(dk_pool* pool, int32_t reset, double* us_out, int64_t* calls_out);

const char* dk_strerror(int32_t status);
int32_t dk_last_hip_error(dk_pool* pool);

#ifdef __cplusplus
}
#endif
#endif /* DELTAKV_H */
