/*
 * xy_attn.h — C ABI of the attention meta-kernel library for MI355X (gfx950).
 *
 * One matmul-softmax-matmul primitive over fixed-size (Q tile x KV block) work
 * units serves a single mixed batch of prefill chunks, prefix-cached prefill
 * suffixes, single-token decodes and speculative-decoding verify segments, all
 * reading a paged K/V cache through a block table (paper sections 3.2.1, 3.3.1
 * and 4).  The host side turns per-sequence descriptors (the paper's
 * Token-Table) into a sorted, load-balanced flat list of work units per worker
 * (the paper's Task-Table); the device side is a persistent kernel in which
 * every workgroup walks its own list.
 *
 * Conventions
 *   - every function returns an int status (0 = XY_OK, negative = error) unless
 *     stated otherwise; no exception crosses this boundary;
 *   - "host" / "device" says where a pointer must live;
 *   - the library owns only what xy_attn_plan_create / xy_attn_plan_upload
 *     allocate, and frees it in xy_attn_plan_destroy; every tensor belongs to
 *     the caller;
 *   - a call that fails enqueues no device work.
 *   - element type of Q, K, V, O is bf16; strides are in elements; the head
 *     dimension is contiguous.
 */
#ifndef XY_ATTN_H
#define XY_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { XY_OK = 0, XY_ERR_ARG = -1, XY_ERR_DESC = -2, XY_ERR_CAPACITY = -3,
       XY_ERR_WORKSPACE = -4, XY_ERR_HIP = -5, XY_ERR_NOMEM = -6 };

/* Stage kinds of a Token-Table entry (section 3.2.1: P / D / V stages). */
enum { XY_PREFILL = 0, XY_DECODE = 1, XY_VERIFY = 2 };
/* Section 4.1.2: sequence-based speculation keeps the causal corner (mask-free);
 * tree-based speculation passes the specLen x specLen corner explicitly. */
enum { XY_MASK_CAUSAL = 0, XY_MASK_TREE = 1 };

/* One Token-Table entry (section 3.2.1).  The entry's start position in the
 * packed Q / O tensors is implicit: the running sum of query_len. */
typedef struct {
  int32_t query_len;        /* tokenNum: new tokens scheduled this step, >= 1; DECODE: exactly 1 */
  int32_t context_len;      /* historical kvLen: tokens cached before these, >= 0.  The sequence
                               holds context_len + query_len keys; this step's own K/V must
                               already sit in the cache at positions context_len ..           */
  int32_t kind;             /* XY_PREFILL | XY_DECODE | XY_VERIFY */
  int32_t mask_kind;        /* XY_MASK_TREE only with XY_VERIFY and query_len <= 64 */
  int64_t mask_word_offset; /* first uint32 word of this sequence's packed corner mask; ignored
                               unless XY_MASK_TREE.  Row r occupies ceil(query_len/32) words,
                               little-endian; bit s of row r set = query r may see key
                               context_len + s.  Keys below context_len are always visible
                               (section 4.1.2).                                               */
} xy_seq_desc;

/* Plan parameters.  tile sizes are the paper's per-stage tileSize (section
 * 3.2.1); num_workers is the number of "cores" of the Task-Table (section 3.3). */
typedef struct {
  int32_t num_q_heads;            /* Hq */
  int32_t num_kv_heads;           /* Hkv, divides Hq; query head h reads KV head h / (Hq/Hkv) */
  int32_t head_dim;               /* must be 128 */
  int32_t block_size;             /* tokens per KV block (page): 16, 32, 64 or 128 */
  int32_t max_blocks_per_seq;     /* row stride of the block table, in blocks of block_size tokens */
  int32_t num_workers;            /* W >= 1: persistent workgroups */
  int32_t prefill_tile_tokens;    /* tokens per PREFILL unit */
  int32_t prefill_heads_per_unit; /* heads per PREFILL unit; divides Hq/Hkv */
  int32_t verify_tile_tokens;     /* tokens per DECODE / VERIFY unit (these always take the
                                     Hq/Hkv heads of one KV head); XY_TILE_AUTO = chosen per
                                     sequence (see XY_TILE_AUTO)                             */
  int32_t split_kv_blocks;        /* a DECODE / VERIFY unit visiting more 128-key K/V tiles than this
                                     is split along K/V; 0 = never; XY_SPLIT_AUTO = chosen per
                                     batch (see XY_SPLIT_AUTO)                                */
  int32_t cost_row_floor;         /* load = max(rows, floor) * tiles; 1 = the paper's
                                     tileSize x kvLen (section 3.3.1) in units of 128 keys   */
  int32_t assign_policy;          /* XY_ASSIGN_SNAKE: the paper's symmetric round-robin over the
                                     sorted units (section 3.3.1); XY_ASSIGN_LEAST_LOADED: each
                                     sorted unit goes to the worker with the smallest load so far
                                     (lowest index on ties); XY_ASSIGN_DYNAMIC: units of more
                                     than 32 rows as with XY_ASSIGN_LEAST_LOADED (among
                                     themselves), units of at most 32 rows are not assigned at
                                     all: they form one list in sorted order behind the workers'
                                     lists (worker_offsets[W] is where it starts) and the
                                     wavefronts of all workers draw from it at run time; when
                                     there is nothing to even out (no unit of more than 32 rows
                                     and all loads equal) or nothing worth it (no unit of more
                                     than 32 rows and none that visits more than 2 K/V tiles: a
                                     draw from the shared cursor takes about as long as such a
                                     unit) the plan is XY_ASSIGN_LEAST_LOADED's.
                                     A plan with a shared list keeps its cursor in device memory
                                     of its own: one xy_attn_run of it at a time                */
} xy_attn_config;

/* split_kv_blocks = XY_SPLIT_AUTO: the K/V split (this design's extension of the Update stage of section
 * 4.2.1 across workers) is sized to the batch.  Units of at most 32 rows are processed one per wavefront,
 * L = 4 * num_workers wavefronts in all.  Let F be the number of DECODE / VERIFY families of at most 32
 * rows (token tiles x KV heads) and nb the number of 128-key tiles a family visits.
 *  - All such families visit the same nb: each is cut into k pieces, k minimising
 *    ceil(F k / L) * (ceil(nb / k) + 1) (rounds of wavefront slots x tiles per piece, a piece costing about
 *    one tile on top of its own for set-up, partial result and merge) over k = 1 .. nb, the smallest such
 *    k on ties; the split size is ceil(nb / k).
 *  - Otherwise, with s = ceil(B / L) one wavefront's share of the tiles B of all these families together, the
 *    split size is min(max(s, 2), max(16, min(64, floor(2 s / 5)))): the share itself for small batches, 16
 *    tiles up to a share of 40, then two fifths of the share (about three pieces per wavefront, which the shared
 *    list still evens out, each piece costing about a tile and a half beyond its own), at most 64.
 * DECODE / VERIFY families of more than 32 rows are split at 16 tiles.  A batch with fewer families of more
 * than 32 rows than workers, U < num_workers, and little else to do (a prefill chunk with no or few decodes
 * beside it: 2 N < M (num_workers - U), N the summed load max(rows, cost_row_floor) x nb of the families of at
 * most 32 rows, M the largest load of a wide family) has each wide family cut at
 * max(8, ceil(nb / floor(num_workers / U))) tiles, PREFILL families included (elsewhere a PREFILL family is
 * never cut). */
#define XY_SPLIT_AUTO (-1)
/* verify_tile_tokens = XY_TILE_AUTO: a DECODE / VERIFY sequence is tiled in 32 / G tokens (G = Hq / Hkv: units of 32
 * rows, one wavefront each), except a sequence with more query tokens than that which visits at least 32 K/V tiles
 * (4096 keys): its narrow tiles would each stream the same K/V, so it is tiled in min(query_len, 256 / G) tokens
 * instead, i.e. one wide unit per KV head for a draft of up to 256 / G tokens. */
#define XY_TILE_AUTO (-1)
enum { XY_ASSIGN_SNAKE = 0, XY_ASSIGN_LEAST_LOADED = 1, XY_ASSIGN_DYNAMIC = 2 };
/* Placement of the units of more than 32 rows under XY_ASSIGN_LEAST_LOADED and XY_ASSIGN_DYNAMIC when 8 divides
 * num_workers (this design; the paper's "cores" of section 3.3 share one cache, the 8 chiplets of this GPU each
 * have an L2 of their own, and workers [x W / 8, (x + 1) W / 8) run on chiplet x): the units of one
 * (sequence, KV head) - all its token tiles and head groups, which read the same K/V - form a group; the groups,
 * by summed load descending (ties: sequence, KV head ascending), go to the chiplet with the smallest load so far
 * (lowest index among equals); a unit goes to the least-loaded worker of its group's chiplet.  If the heaviest
 * chiplet ends more than 3 % above the mean load (max * 8 * 100 > total * 103) no groups are used and every
 * unit goes to the least-loaded worker overall. */
/* rows = tile tokens x heads per unit must be <= 256 for every kind. */

/* One tiling unit (section 3.2.1) placed in the Task-Table (section 3.3.1). */
typedef struct {
  int32_t seq;                    /* index into the descriptor array */
  int32_t head_begin, head_count; /* query heads [head_begin, head_begin + head_count) */
  int32_t q_begin, q_count;       /* query rows of that sequence */
  int32_t kv_block_begin, kv_block_end; /* K/V tiles of 128 keys visited (mask-aware, section 4.2.2); a
                                           tile is 128 / block_size consecutive block-table entries */
  int32_t split_index, num_splits;      /* position among the K/V splits of its family */
  int32_t kind_flags;             /* kind | mask_kind << 2 */
  int64_t cost;                   /* load used for sorting */
  int64_t ws_offset;              /* fp32 element offset of this unit's partial in the workspace,
                                     -1 when the family is not split */
} xy_work_unit;

/* One family of K/V-split units whose partial results must be merged
 * (section 4.2.1, the Update stage's running max / sum, applied across units). */
typedef struct {
  int32_t seq, head_begin, head_count, q_begin, q_count, num_splits;
  int64_t ws_offset;              /* slab base: num_splits x [rows x head_dim acc | rows m | rows l] fp32 */
} xy_merge_item;

typedef struct xy_attn_plan xy_attn_plan; /* opaque, library-owned */

/* Fill *out with the default parameters for a head shape: one unit per KV head
 * with 256 rows for prefill, decode / verify tiles chosen per sequence (XY_TILE_AUTO: 32 / (Hq/Hkv) tokens,
 * the bandwidth-bound unit shape of the kernel, or a whole long-context segment), 256 workers, K/V
 * split sized to the batch (XY_SPLIT_AUTO), cost floor 128, dynamic assignment.  Host only. */
int xy_attn_default_config(int32_t num_q_heads, int32_t num_kv_heads, int32_t max_blocks_per_seq,
                           xy_attn_config* out /* host */);

/* Decompose (section 3.2.1), cost, sort (section 3.3.1) and assign to the workers by cfg->assign_policy (the
 * paper's symmetric round-robin is XY_ASSIGN_SNAKE; the default is XY_ASSIGN_DYNAMIC).
 * Host only, integers only, deterministic; touches no GPU.
 * descs: host array of num_seqs entries (num_seqs = 0 gives an empty plan).
 * Errors: XY_ERR_ARG (null pointer, bad head shape, more than 256 query heads per KV head, head_dim != 128,
 * block_size not 16/32/64/128, rows > 256, non-positive parameter, unknown assign_policy), XY_ERR_DESC
 * (query_len < 1, negative context, DECODE with query_len != 1, TREE on a non-VERIFY entry or with more
 * than 64 tokens, unknown kind), XY_ERR_CAPACITY (a sequence needs more than max_blocks_per_seq
 * blocks, or more than 2^31-1 tokens or units in total). */
int xy_attn_plan_create(const xy_attn_config* cfg /* host */, const xy_seq_desc* descs /* host */,
                        int32_t num_seqs, xy_attn_plan** out /* host */);

/* Borrowed host pointers, valid until xy_attn_plan_destroy.  units are grouped
 * by worker: worker w owns units[worker_offsets[w] .. worker_offsets[w+1]).
 * Any output pointer may be NULL. */
int xy_attn_plan_get(const xy_attn_plan* plan, const xy_work_unit** units, int64_t* num_units,
                     const int32_t** worker_offsets /* W + 1 entries */,
                     const xy_merge_item** merges, int64_t* num_merges);

/* Bytes of device workspace xy_attn_run needs for this plan (0 if nothing is split).
 * The workspace needs no initialisation; runs that may overlap in time need separate ones. */
int xy_attn_plan_workspace_bytes(const xy_attn_plan* plan, size_t* bytes /* host */);

/* The same for the next batch in an existing plan object (a serving loop plans every step): the object keeps
 * its host buffers and its memory on the GPU, so nothing is allocated or freed unless the new plan is larger
 * than any before it.  cfg may differ from the one the plan was created with.  The arguments are validated
 * before the plan is touched (errors as for xy_attn_plan_create: the old plan stays as it was); if host memory
 * runs out (XY_ERR_NOMEM) the plan is left empty.  Pointers handed out by xy_attn_plan_get are invalidated.  No
 * run of the old plan may still be in flight on a stream other than the one the next copy or run is given. */
int xy_attn_plan_rebuild(xy_attn_plan* plan, const xy_attn_config* cfg /* host */, const xy_seq_desc* descs /* host */,
                         int32_t num_seqs);

/* Copy the plan's tables to the current HIP device.  The plan owns one device arena and one pinned staging
 * buffer of the same size (allocated on first use, grown only when a rebuilt plan does not fit, freed by
 * xy_attn_plan_destroy); a copy packs the tables into the staging buffer and enqueues one small kernel that
 * reads it from there (a kernel, not a copy-engine transfer: handing a stream from the copy engine to the next
 * kernel costs more than such a step may take).
 *   xy_attn_plan_upload        on the default stream, and waits for it;
 *   xy_attn_plan_upload_async  on hip_stream, without waiting: work enqueued on that stream afterwards sees
 *                              the tables; work on other streams must be ordered behind it by the caller.
 * Both return at once when the tables on the GPU are current.  Optional: xy_attn_run, xy_attn_append_kv and
 * xy_attn_run_fused_qkv do the asynchronous copy on their own stream when the plan is new or was rebuilt.
 * Errors: XY_ERR_ARG (null; the plan's arena lives on another device), XY_ERR_HIP. */
int xy_attn_plan_upload(xy_attn_plan* plan);
int xy_attn_plan_upload_async(xy_attn_plan* plan, void* hip_stream);

/* Enqueue the whole batch on hip_stream (a hipStream_t, NULL = default stream)
 * and return without waiting.
 *   q            device, bf16, element (t, h, d) at q[t*q_token_stride + h*q_head_stride + d],
 *                t = packed token index in descriptor order (may alias a fused QKV tensor)
 *   k_cache, v_cache  device, bf16, element (block, kv_head, slot, d) at
 *                block*kv_block_stride + kv_head*kv_head_stride + slot*kv_token_stride + d.
 *                Whole blocks are read; slots past a sequence's length may hold any bit pattern
 *                (NaN and infinities included: memory that was never written) and do not
 *                influence the result (section 5.2: padded keys are neutralised in the softmax;
 *                here their scores are overwritten and their V rows cleared on chip).  Only the
 *                first ceil((context_len + query_len) / block_size) table entries of a sequence
 *                are ever dereferenced.
 *   block_table  device, int32 [num_seqs][max_blocks_per_seq] physical block ids (section 4.1.1)
 *   tree_masks   device, packed corner masks; may be NULL when no entry is XY_MASK_TREE
 *   out          device, bf16, laid out like q with its own strides; every scheduled
 *                (token, head) row is overwritten, nothing else is written
 *   workspace    device, >= xy_attn_plan_workspace_bytes, 16-byte aligned; may be NULL if 0
 *   softmax_scale  finite, > 0
 * Only a call that has to copy a new or rebuilt plan to the GPU first (no xy_attn_plan_upload before it) may
 * allocate, and only when the plan's arena is missing or too small.
 * Rows with no visible key are written as zeros.
 * Errors: XY_ERR_ARG, XY_ERR_WORKSPACE (too small / misaligned), XY_ERR_HIP. */
int xy_attn_run(xy_attn_plan* plan,
                const void* q, int64_t q_token_stride, int64_t q_head_stride,
                const void* k_cache, const void* v_cache,
                int64_t kv_block_stride, int64_t kv_head_stride, int64_t kv_token_stride,
                const int32_t* block_table, const uint32_t* tree_masks,
                void* out, int64_t o_token_stride, int64_t o_head_stride,
                void* workspace, size_t workspace_bytes,
                float softmax_scale, void* hip_stream);

/* The two launches xy_attn_run is made of, separately (for per-kernel timing with
 * events between them): XY_PHASE_UNITS runs the persistent work-unit kernel
 * (sections 3.3 and 4: every worker walks its Task-Table entry), XY_PHASE_MERGE
 * merges the partial results of K/V-split units (Update stage, section 4.2.1).
 * phases is a bit mask; both bits = xy_attn_run.  The output of a split family
 * is valid only after both phases have run, in this order, with the same
 * arguments.  Same arguments, ownership and errors as xy_attn_run. */
enum { XY_PHASE_UNITS = 1, XY_PHASE_MERGE = 2 };
int xy_attn_run_phase(int phases, xy_attn_plan* plan,
                      const void* q, int64_t q_token_stride, int64_t q_head_stride,
                      const void* k_cache, const void* v_cache,
                      int64_t kv_block_stride, int64_t kv_head_stride, int64_t kv_token_stride,
                      const int32_t* block_table, const uint32_t* tree_masks,
                      void* out, int64_t o_token_stride, int64_t o_head_stride,
                      void* workspace, size_t workspace_bytes,
                      float softmax_scale, void* hip_stream);

/* Write this step's K and V rows into their paged slots, so that the cache holds "both historical
 * and newly generated" tokens when xy_attn_run reads it (section 4.1.1).  New token r of sequence i
 * (packed token index t_i + r) goes to key position context_len + r: physical block
 * block_table[i][(context_len + r) / block_size], slot (context_len + r) % block_size, for every KV head; nothing
 * else in the cache is written.  Bit patterns are copied, never converted.
 *   k_new, v_new  device, bf16, element (t, g, d) at x_new[t*new_token_stride + g*new_head_stride + d],
 *                 g = KV head.  They may point into one fused projection output
 *                 [tokens, Hq + 2 Hkv, 128] (section 5: read in place by stride, no split / permute)
 *   k_cache, v_cache, strides, block_table  as for xy_attn_run, but written here
 * Enqueues one launch on hip_stream and returns without waiting; a later xy_attn_run on the same
 * stream sees the rows.  Two sequences that share a block may not both append into it (the shared
 * prefix blocks of section 4.1.1 are full blocks; a partial block is private).
 * Errors: XY_ERR_ARG (null pointer, stride not a multiple of 8 elements or base not 16-byte aligned,
 * wrong device), XY_ERR_HIP.  An empty plan is a no-op. */
int xy_attn_append_kv(xy_attn_plan* plan,
                      const void* k_new, const void* v_new, int64_t new_token_stride, int64_t new_head_stride,
                      void* k_cache, void* v_cache,
                      int64_t kv_block_stride, int64_t kv_head_stride, int64_t kv_token_stride,
                      const int32_t* block_table, void* hip_stream);

/* xy_attn_append_kv followed by xy_attn_run on one fused projection output (section 5):
 *   qkv  device, bf16, [tokens][Hq + 2 Hkv][128] with the given token and head strides; heads
 *        0 .. Hq-1 are Q, the next Hkv are K, the last Hkv are V.
 * Q is read in place, K and V rows are scattered into the cache first, then attention runs on the
 * same stream.  Other arguments, ownership and errors as for the two calls it is made of. */
int xy_attn_run_fused_qkv(xy_attn_plan* plan,
                          const void* qkv, int64_t qkv_token_stride, int64_t qkv_head_stride,
                          void* k_cache, void* v_cache,
                          int64_t kv_block_stride, int64_t kv_head_stride, int64_t kv_token_stride,
                          const int32_t* block_table, const uint32_t* tree_masks,
                          void* out, int64_t o_token_stride, int64_t o_head_stride,
                          void* workspace, size_t workspace_bytes,
                          float softmax_scale, void* hip_stream);

/* xy_attn_run for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  The partial results of K/V-split units go to
 * a fixed array of XY_STATIC_WORKSPACE_BYTES in device memory that is part of the library (every GPU the library
 * runs on holds its own copy until the process ends); the call itself allocates nothing and calls no allocating
 * routine.  Same arguments, ownership, output and errors as xy_attn_run, without the workspace, and:
 *   - the plan's current tables must already be on the GPU (xy_attn_plan_upload / _async, or an earlier
 *     xy_attn_run, after the last rebuild): XY_ERR_ARG otherwise;
 *   - a plan that needs more than XY_STATIC_WORKSPACE_BYTES (xy_attn_plan_workspace_bytes) is refused with
 *     XY_ERR_WORKSPACE and nothing is enqueued;
 *   - all calls on one GPU share that GPU's array, which keeps what the last call left there (nothing has to be
 *     cleared: every split unit writes its whole partial result before the merge pass reads it); calls that may
 *     overlap in time on one GPU (two streams, two threads) race on it and must be serialised by the caller. */
#define XY_STATIC_WORKSPACE_BYTES (64 * 1024 * 1024)
int xy_attn_run_static(xy_attn_plan* plan,
                       const void* q, int64_t q_token_stride, int64_t q_head_stride,
                       const void* k_cache, const void* v_cache,
                       int64_t kv_block_stride, int64_t kv_head_stride, int64_t kv_token_stride,
                       const int32_t* block_table, const uint32_t* tree_masks,
                       void* out, int64_t o_token_stride, int64_t o_head_stride,
                       float softmax_scale, void* hip_stream);

/* Copy-on-write of a partly reused block (section 4.1.1): rows [0, rows) of block src_block are
 * copied to block dst_block, K and V, every KV head. */
typedef struct {
  int32_t src_block, dst_block, rows;
} xy_kv_copy;

/* Run n such copies on hip_stream (before the step that appends to the destination blocks).  The copies of one
 * call run side by side: no destination block of a call may be the source or the destination of another copy
 * of the same call (order dependent copies by separate calls on one stream).
 *   copies  host array; its content is captured by the call
 *   caches and strides as for xy_attn_run; num_kv_heads >= 1; rows <= the block size in use
 * Errors: XY_ERR_ARG (null pointer, n < 0, rows < 0, stride / alignment as for xy_attn_run), XY_ERR_HIP. */
int xy_attn_copy_block_rows(const xy_kv_copy* copies /* host */, int32_t n, int32_t num_kv_heads,
                            void* k_cache, void* v_cache,
                            int64_t kv_block_stride, int64_t kv_head_stride, int64_t kv_token_stride,
                            void* hip_stream);

/* Free host and device memory of the plan (NULL is allowed). */
void xy_attn_plan_destroy(xy_attn_plan* plan);

/* Static string for a status code. */
const char* xy_attn_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* XY_ATTN_H */
