/*
 * xy_serve.h — C ABI of the host-side producers of the attention inputs.
 *
 * Two pieces of the paper's serving loop decide what the attention kernel is asked
 * to do each step: the token-wise scheduler (section 3.1) that fills a fixed token
 * budget with prefill, decode and speculative tokens, cutting long prompts, and
 * the K/V block manager (section 4.1.1): a radix tree of cache blocks with
 * token-wise prefix reuse, copy-on-write for a block that matches in part, and
 * eviction of the least recently used leaves.  Both are host code, integers
 * only, deterministic; they touch no GPU.  Their outputs are what xy_attn.h
 * consumes: xy_seq_desc entries (query_len, context_len, kind) and block-table
 * rows, plus the row copies (xy_kv_copy) to run before the step.
 *
 * Every function returns an int status from xy_attn.h (0 = XY_OK).
 */
#ifndef XY_SERVE_H
#define XY_SERVE_H

#include "xy_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---- token-wise scheduling (section 3.1) ------------------------------------------------- */

typedef struct {
  int32_t request;      /* caller's id, unique in the queue */
  int32_t kind;         /* XY_PREFILL | XY_DECODE | XY_VERIFY */
  int32_t tokens;       /* PREFILL: rest of the prompt; DECODE: 1; VERIFY: draft length; >= 1 */
  int32_t context_len;  /* tokens of this request already in the cache */
} xy_queue_entry;

typedef struct {
  int32_t request, kind;
  int32_t query_len;    /* tokens scheduled this step (a prefill may be cut, nothing else is) */
  int32_t context_len;
} xy_chunk_entry;

/* Compose one chunk of at most token_budget tokens from the queue (arrival order).
 *  1. decode / verify entries receive slots, in queue order, while the slots handed out stay within
 *     reserved_decode_slots ("certain slots are reserved for decode and speculative tokens"); an entry
 *     that does not fit there is passed over (a verify segment is never cut);
 *  2. prefill entries, in queue order, receive the rest of the budget ("prefill requests are
 *     prioritized"); the first that does not fit whole is cut to what is left and ends the pass;
 *  3. budget still left goes to the entries passed over in 1, in queue order, while they fit.
 * chunk (host, capacity n) receives the chosen entries: prefill first, then decode / verify, each in
 * queue order.  Errors: XY_ERR_ARG (null pointer, negative count, budget < 1, reserve outside
 * [0, budget], an entry with tokens < 1, negative context or unknown kind, a decode with tokens != 1). */
int xy_serve_schedule_chunk(int32_t token_budget, int32_t reserved_decode_slots,
                            const xy_queue_entry* queue /* host */, int32_t n,
                            xy_chunk_entry* chunk /* host, capacity n */, int32_t* num_chunk /* host */);

/* ---- K/V block manager (section 4.1.1) --------------------------------------------------- */

typedef struct xy_kv_manager xy_kv_manager; /* opaque, library-owned */

/* num_blocks physical blocks of block_size tokens, all free (handed out in ascending id). */
int xy_kv_create(int32_t num_blocks, int32_t block_size, xy_kv_manager** out /* host */);
void xy_kv_destroy(xy_kv_manager* m);

/* Admit a prompt.  Walks the tree while whole blocks match and at least one token is left to compute,
 * then reuses the longest common prefix (>= 1 token, lowest block id among equals) of one more block
 * through copy-on-write: a private block is allocated and *copy says which rows to copy into it
 * (*num_copies = 1), the shared block is never written.  The sequence then holds *cached_tokens
 * tokens; the caller extends it with the rest of the prompt.  The reused blocks are pinned.
 * Errors: XY_ERR_ARG (null pointer, n < 1), XY_ERR_CAPACITY (no block could be had; nothing changed). */
int xy_kv_open(xy_kv_manager* m, const int32_t* tokens /* host */, int32_t n, int32_t* seq /* host */,
               int32_t* cached_tokens /* host */, xy_kv_copy* copy /* host */, int32_t* num_copies /* host */);

/* Append n tokens to a sequence (their K/V rows are written by the step that runs them).  Allocates
 * blocks as needed -- lowest free id, else the least recently used unpinned leaf of the tree is
 * evicted -- and inserts every private block that becomes full into the tree below the sequence's
 * last tree block, pinned by this sequence (if a block with the same tokens is already there, the
 * sequence keeps its own blocks private from then on).
 * Errors: XY_ERR_ARG (unknown sequence, null pointer, n < 0), XY_ERR_CAPACITY (not enough blocks:
 * the sequence is unchanged; leaves evicted for the attempt stay evicted, their blocks are free). */
int xy_kv_extend(xy_kv_manager* m, int32_t seq, const int32_t* tokens /* host */, int32_t n);

/* Block-table row of a sequence: ceil(length / block_size) physical block ids.  row may be NULL to
 * query the sizes.  Errors: XY_ERR_ARG (unknown sequence, capacity too small). */
int xy_kv_block_row(const xy_kv_manager* m, int32_t seq, int32_t* row /* host */, int32_t capacity,
                    int32_t* num_blocks /* host */, int32_t* length /* host, tokens */);

/* Finish a sequence: its tree blocks are unpinned and stay cached, its private blocks become free. */
int xy_kv_close(xy_kv_manager* m, int32_t seq);

/* out[0] free blocks, out[1] blocks in the tree, out[2] evictions so far, out[3] open sequences. */
int xy_kv_stats(const xy_kv_manager* m, int64_t out[4] /* host */);

#ifdef __cplusplus
}
#endif
#endif /* XY_SERVE_H */
