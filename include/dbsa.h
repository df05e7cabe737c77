/*
 * dbsa.h -- C ABI of libdbsa: block-sparse causal attention over a demonstration
 * KV cache (Dynamic Block-Sparse Attention), for AMD MI355X (gfx950).
 *
 * Vocabulary.  The paper calls the unit of encoding and retrieval a "block" of k
 * demonstrations (Sec. 2.1).  Here that unit is a GROUP; "KV tile" / "Q tile" are
 * kernel tiles of tokens.  Token order of a pool: the attention-sink prefix
 * [0, S), then the demonstrations; groups are runs of whole demonstrations.
 *
 * All tensors are token-major [tokens, heads, D] with the D elements of one
 * (token, head) contiguous; strides are given in ELEMENTS.  For dbsa_preencode_attn,
 * dbsa_query_attn, dbsa_decode_attn and dbsa_decode_attn_kv8 Q/K/V are post-RoPE:
 * these calls never apply positions, so the K handed to the query stage may be a
 * re-positioned copy (Sec. 2.2) of the K used at pre-encoding.  The *_rope calls
 * apply the new in-order position ids of Sec. 2.2 themselves (see there).
 *
 * Every function returns DBSA_OK (0) or a negative error code; nothing throws
 * across the boundary.  Functions are thread-safe on distinct layouts.  The
 * attention entry points only enqueue work on the caller's stream and never
 * synchronise it; neither do dbsa_layout_build and dbsa_layout_destroy.  The
 * caller owns every tensor and the workspace; the library owns only dbsa_layout
 * objects (build / destroy) and the device blocks their lists live in.
 */
#ifndef DBSA_H_
#define DBSA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  DBSA_OK = 0,
  DBSA_ERR_INVALID_ARG = -1,   /* null pointer, non-positive size, misaligned tensor, layout of the wrong stage */
  DBSA_ERR_BAD_BOUNDS = -2,    /* demo/group/query offsets not strictly increasing or not anchored as documented */
  DBSA_ERR_BAD_SELECTION = -3, /* group index out of range, or a group listed twice by one query */
  DBSA_ERR_UNSUPPORTED = -4,   /* head_dim, head ratio, dtype or tile size the kernels do not implement */
  DBSA_ERR_WORKSPACE = -5,     /* workspace missing or smaller than dbsa_workspace_bytes() */
  DBSA_ERR_HIP = -6            /* a HIP runtime call failed; hipGetLastError() holds the cause */
};

enum { DBSA_BF16 = 0, DBSA_F32 = 1 };

/* dbsa_layout_build flag: build the host lists only and touch no GPU.  Such a
 * layout can be exported and destroyed but not passed to an attention call. */
enum { DBSA_LAYOUT_HOST_ONLY = 1 };

/* KV-tile kinds stored in list entries. */
enum {
  DBSA_TILE_FULL = 0,        /* pool keys, every (row, key) pair visible                       */
  DBSA_TILE_CAUSAL = 1,      /* pool keys, pair visible iff key token <= row token             */
  DBSA_TILE_SELF_FULL = 2,   /* keys from the query's own K/V tensor, every pair visible       */
  DBSA_TILE_SELF_CAUSAL = 3  /* own keys, pair visible iff key token <= row token              */
};

/* Static, NUL-terminated description of an error code; never freed. */
const char* dbsa_strerror(int code);

/*
 * The demonstration pool (Sec. 2.1: D is partitioned into groups of whole
 * demonstrations; the first unit is the anchor every group attends).  Host
 * pointers, read during the call only.
 */
typedef struct {
  int32_t sink_len;                  /* S >= 0: tokens [0, S) are the anchor / attention sink               */
  int32_t n_demos;                   /* >= 1                                                                  */
  const int32_t* demo_offsets;       /* [n_demos+1] token offsets; [0] == S; strictly increasing; last == N   */
  int32_t n_groups;                  /* >= 1                                                                  */
  const int32_t* group_demo_offsets; /* [n_groups+1] demo indices; [0] == 0; strictly increasing; last == n_demos */
  int32_t prev_window;               /* number of preceding groups a group attends at pre-encoding (the paper's j);
                                        0 = sink + own group only                                            */
} dbsa_pool_desc;

/*
 * Per-query group selections (Sec. 2.2: a retriever picks a subset of groups for
 * each test query; the anchor is always included and is NOT listed here).  Host
 * pointers, read during the call only.  An empty selection is valid (sink + self).
 */
typedef struct {
  int32_t n_queries;        /* B >= 1                                                                     */
  const int32_t* cu_qlens;  /* [B+1] offsets of each query's prompt tokens in the packed query tensors;
                               [0] == 0; strictly increasing                                              */
  const int32_t* sel_ptr;   /* [B+1] CSR row pointers into sel_idx; [0] == 0; non-decreasing              */
  const int32_t* sel_idx;   /* selected group indices; the caller's order is kept in the lists            */
  int32_t n_split;          /* decode: KV splits per (query, KV head); 0 = let the library choose          */
  const int32_t* page_start;/* NULL: k_pool / v_pool hold the pool contiguously, token j at row j.  Else
                               [n_groups+1]: the row, in the k_pool / v_pool tensors handed to the query
                               and decode calls, of the first token of the sink (index 0) and of group g
                               (index g+1), each segment contiguous from there -- groups live in pages of
                               an arena and may be offloaded or re-encoded independently (Sec. 4, storage
                               cost).  -1 = not resident: selecting such a group is BAD_SELECTION; resident
                               pages that overlap are BAD_BOUNDS.  The lists then name arena rows; position
                               data (dbsa_layout_export_positions) keeps referring to pool token ids.     */
} dbsa_select_desc;

typedef struct dbsa_layout dbsa_layout; /* opaque; owns host and device copies of its index lists */

/*
 * Block-layout builder.  Turns the pool structure (and, if `sel` is non-NULL, the
 * per-query selections) into per-Q-tile lists of KV tiles so that the kernels walk
 * only tiles holding visible keys (Sec. 2.1: masked blocks are skipped).
 *
 *   sel == NULL : pre-encode layout.  Q tiles: the sink segment, then each group,
 *                 cut every block_m tokens from the segment's first token.  List of
 *                 a tile: sink tiles, the tiles of the prev_window preceding groups,
 *                 the own group's tiles up to the diagonal; ascending kv_start.
 *   sel != NULL : query-stage layout.  Q tiles: each query's prompt cut every
 *                 block_m tokens.  List: sink tiles, the tiles of the selected
 *                 groups in the caller's order, then the query's own tiles up to
 *                 the diagonal.  Also builds the decode lists: per query the pool
 *                 part, cut into n_split runs of entries
 *                 [s*L / n_split, (s+1)*L / n_split).
 *
 * KV tiles are cut every block_n tokens inside a segment (sink, group, a query's
 * own tokens) and never straddle segments.  block_m, block_n > 0; the attention
 * calls state which sizes their kernels accept.
 *
 * flags: 0 or DBSA_LAYOUT_HOST_ONLY.  Without HOST_ONLY the lists are copied to
 * the current device with hipMemcpyAsync on `stream` (a hipStream_t, may be
 * NULL); the call does not wait for the copy.  An attention call on another
 * stream is ordered behind the copy by the library (one hipStreamWaitEvent at
 * the layout's first call on that stream).  The device block and its pinned
 * staging twin come from a process-wide pool that dbsa_layout_destroy refills
 * (at most 16 blocks are in flight before a build waits for the oldest one;
 * blocks are kept until the process ends).
 * On success *out receives a layout to be released with dbsa_layout_destroy.
 * Errors: INVALID_ARG, BAD_BOUNDS, BAD_SELECTION, HIP; *out is untouched then.
 */
int dbsa_layout_build(const dbsa_pool_desc* pool, const dbsa_select_desc* sel, int32_t block_m, int32_t block_n,
                      int32_t flags, void* stream, dbsa_layout** out);

/*
 * Pre-encode layout for groups appended to an already encoded pool (Sec. 2.1: a group
 * attends the anchor, its window of preceding groups and itself, and no earlier group
 * attends it, so the cached K/V of the earlier groups stay valid and the encoding cost of
 * an addition does not grow with the pool: Sec. 1, and Sec. 2.1 on adding a block at any time).
 * `pool` describes the WHOLE pool including the new groups; the layout holds the Q tiles
 * of groups first_group .. n_groups-1 only, each with exactly the list the full pre-encode
 * layout gives it.  dbsa_preencode_attn with this layout writes the rows of those groups and
 * leaves every other row of `o` untouched; q/k/v/o are indexed by absolute token as usual.
 * Errors as dbsa_layout_build; first_group outside [0, n_groups) -> INVALID_ARG.
 */
int dbsa_layout_build_append(const dbsa_pool_desc* pool, int32_t first_group, int32_t block_m, int32_t block_n,
                             int32_t flags, void* stream, dbsa_layout** out);

/*
 * Host views of the lists, valid until the layout is destroyed.
 *   qtile_tab : int32 [n_qtiles][4] = (q_start, q_len, owner, 0); owner is -1 for
 *               the sink segment, else the group (pre-encode) or query index.
 *   list_ptr  : int64 [n_qtiles+1] entry offsets.
 *   list_ent  : int32 [n_ent][2] = (kv_start, kv_len | kind << 16).
 * Any output pointer may be NULL.
 */
int dbsa_layout_export(const dbsa_layout* layout, const int32_t** qtile_tab, int64_t* n_qtiles,
                       const int64_t** list_ptr, const int32_t** list_ent, int64_t* n_ent);

/*
 * Decode lists of a query-stage layout (INVALID_ARG for a pre-encode layout).
 *   dec_ptr   : int64 [B+1] offsets of each query's pool entries in dec_ent.
 *   dec_ent   : int32 [n_dec_ent][2], same encoding as list_ent, kinds all FULL.
 *   split_ptr : int64 [B][n_split+1] absolute offsets into dec_ent.
 */
int dbsa_layout_export_decode(const dbsa_layout* layout, const int64_t** dec_ptr, const int32_t** dec_ent,
                              int64_t* n_dec_ent, const int64_t** split_ptr, int32_t* n_split);

/*
 * Re-positioning data of a query-stage layout (INVALID_ARG for a pre-encode layout).
 * Sec. 2.2: the caches of the anchor and of the selected groups are concatenated in the
 * caller's order and receive new in-order position ids 0 .. |D'|-1; the query follows at
 * ids |D'| + a.  The *_rope attention calls expect keys rotated at the id they were ENCODED
 * with (pool keys: their token index, Sec. 2.1 "sequential position ids"; a query's own
 * keys: their index inside the query) and move a run of keys to its new ids by rotating the
 * query row back by the run's displacement instead (rotary scores depend on id differences
 * only), so no per-query copy of the keys is ever made.
 *   list_shift : int32 [n_ent], parallel to list_ent.  Row number i of a Q tile (i = 0 at the
 *                tile's first row) scores the keys of entry e after a rotation at id
 *                list_shift[e] + i.
 *   qref_shift : int32 [n_qrefs], parallel to qrefs of the group-major decode schedule: the
 *                decode row of query u scores the item's keys after a rotation at id
 *                qref_shift[ref] + self_len[u] - 1; its own cached keys at self_len[u] - 1.
 *   cache_len  : int32 [B] = |D'| of each query (sink + selected groups).
 * Any output pointer may be NULL; views are valid until the layout is destroyed.
 */
int dbsa_layout_export_positions(const dbsa_layout* layout, const int32_t** list_shift, const int32_t** qref_shift,
                                 const int32_t** cache_len);

/*
 * Group-major decode schedule of a query-stage layout (INVALID_ARG for a pre-encode
 * layout).  Queries that selected the same group read the same KV (Sec. 2.2: the caches
 * of the selected groups are reused in place), so one work item covers a run of KV tiles
 * of one segment for up to 32 of the queries that use it; each (item, query) pair owns one
 * partial-softmax slot and the last slot of a query is for its own cached keys.
 *   seg_ptr   : int64 [n_groups+2]: tile offsets of the sink (segment 0) and of group g
 *               (segment g+1) in seg_ent.
 *   seg_ent   : int32 [n_seg_ent][2], same encoding as list_ent, kinds all FULL.
 *   items     : int32 [n_items][4] = (ent_begin, ent_count, qref_begin, n_q).  Order:
 *               segments ascending (those with a user), runs ascending (a segment of t
 *               tiles is cut into n = ceil(t / chunk_tiles) runs of equal length to within
 *               one tile, run i = tiles [i t / n, (i+1) t / n)), users in ascending query
 *               order in batches of 32.  The sink's users are all queries.
 *   qrefs     : int32 [n_qrefs][2] = (query, slot).
 *   slot_ptr  : int64 [B+1]: slots of query u are slot_ptr[u] .. slot_ptr[u+1]-1, numbered
 *               in item order; the last one is the own-cache slot.
 *   chunk_tiles: most tiles per run: ceil(longest segment with a user / n_split) when the
 *               caller gave n_split > 0, else chosen by the library (at most 32).
 */
int dbsa_layout_export_decode_groups(const dbsa_layout* layout, const int64_t** seg_ptr, const int32_t** seg_ent,
                                     int64_t* n_seg_ent, const int32_t** items, int64_t* n_items,
                                     const int32_t** qrefs, int64_t* n_qrefs, const int64_t** slot_ptr,
                                     int32_t* chunk_tiles);

/* Launch order of Q tiles: a permutation of [0, n_qtiles), owner by owner, the longest list
 * of an owner first. */
int dbsa_layout_export_order(const dbsa_layout* layout, const int32_t** order, int64_t* n_order);

/*
 * Schedule of a persistent prefill-shaped launch (plumbing of the launches, not an operation of
 * the paper): large launches run as many workgroups as the chip holds, n_classes of them per
 * block of query heads, and worker c walks the Q tiles records[4 * class_ptr[c]] ..
 * records[4 * class_ptr[c+1]) one after the other, four int32 each: (q_start, q_len, first list
 * entry, list entries).  Every Q tile appears exactly once.  Tiles are dealt in launch order in
 * rounds of n_classes, the longest list of a round to the worker with the least work so far (work
 * of a tile = its list entries + 3).  A layout keeps ONE schedule, fixed by the first call that
 * needs one (this call or an attention call): INVALID_ARG for another n_classes later, for
 * n_classes outside [1, 512] or a NULL layout.  The arrays belong to the layout.
 */
int dbsa_layout_export_schedule(const dbsa_layout* layout, int32_t n_classes, const int32_t** class_ptr,
                                const int32_t** records);

/*
 * The records of a decode step that runs as a contraction (plumbing; query-stage layouts): record i =
 * four int32 (first reference, references, first tile, tiles): at most 64 queries over the tiles
 * seg_ent[first tile .. + tiles) of one run of one segment.  row_fill = share of the 64 rows of a
 * record that carry a query, weighted by tiles: a decode step with query heads in fours per KV head and
 * row_fill >= 0.22 (with or without re-positioning) runs these records as a dense contraction (64
 * queries per wavefront) instead of the 32-column work items, into partial states that the same merge
 * combines.
 * Below that fill the records are the work items' runs taken in pairs: the references are qrefs of
 * dbsa_layout_export_decode_groups and every (item, query) pair appears in exactly one record with
 * the slot it has there.  From that fill on the records have runs, references and slots of their own,
 * see dbsa_layout_export_matrix_plan.  The array belongs to the layout.  Errors: INVALID_ARG.
 */
int dbsa_layout_export_matrix_records(const dbsa_layout* layout, const int32_t** records, int64_t* n_records,
                                      float* row_fill);

/*
 * How a layout with row_fill >= 0.22 cuts and deals the records above (plumbing).  At build time the
 * (segment, 64 queries) units are walked in order and dealt to `nominal_workers` = compute units / 8
 * workers per KV head (fewer when a worker's share would hold under 12 tiles), each taking tiles until
 * its cost (tiles + 4.5 per run) reaches the share; a unit that does not fit is cut there, no run is
 * shorter than 4 tiles.  Worker c of a step whose compute units per head block equal nominal_workers
 * takes records plan_ptr[c] .. plan_ptr[c+1]-1 (n_workers + 1 entries); a step with another worker
 * count deals the same records at launch.  qrefs: int32 [n_qrefs][2] = (query, slot), the references
 * of the records; slot_ptr: int64 [B+1], slots of query u are slot_ptr[u] .. slot_ptr[u+1]-1 in
 * record order, the last one its own-cache slot (a contraction step uses these slots, every other step
 * those of dbsa_layout_export_decode_groups; dbsa_workspace_bytes covers both).  Layouts below that
 * fill have no plan: n_workers = 0, n_qrefs = 0.  The arrays belong to the layout.  Errors: INVALID_ARG.
 */
int dbsa_layout_export_matrix_plan(const dbsa_layout* layout, const int32_t** plan_ptr, int32_t* n_workers,
                                   int32_t* nominal_workers, const int32_t** qrefs, int64_t* n_qrefs,
                                   const int64_t** slot_ptr);

/*
 * Device blocks (each with a pinned host twin) that hold the lists of destroyed layouts and wait
 * to be reused by a later dbsa_layout_build (plumbing).  At most 16 are kept: idle blocks beyond
 * that are freed, oldest first, when a layout is destroyed or a build has to allocate.
 */
int32_t dbsa_pooled_list_blocks(void);

/* NULL is allowed.  Does not wait for the device: it may be called right after the last launch
 * that uses the layout.  The device lists stay intact until every stream the layout was used on
 * has passed the point of this call (one event per such stream is recorded here, so those
 * streams must still exist and must not be under graph capture); only then does a later
 * dbsa_layout_build reuse the block.  If an event cannot be recorded the call falls back to
 * hipDeviceSynchronize.  A HIP graph that recorded calls on the layout refers to its device lists:
 * it must not be replayed after this call. */
void dbsa_layout_destroy(dbsa_layout* layout);

/*
 * Bytes of device workspace the query-stage calls use for this layout: one partial softmax
 * state of (head_dim + 4) floats per query head and slot.  dbsa_decode_attn needs the larger
 * of its two schedules (B * n_split slots, or slot_ptr[B] slots).  dbsa_query_attn may use up
 * to 4 slots per query token when the layout has so few Q tiles that the launch would leave
 * compute units idle; it then cuts every KV list into runs and merges their partial states
 * (without a workspace it runs every list in one pass: same result up to summation order).
 * The pre-encode call needs none.  Returns 0 for a pre-encode layout.
 */
size_t dbsa_workspace_bytes(const dbsa_layout* layout, int32_t n_q_heads, int32_t head_dim);

/* A device tensor [tokens, heads, D]: element strides between tokens and heads. */
typedef struct {
  const void* ptr;     /* device pointer, 16-byte aligned            */
  int64_t stride_tok;  /* elements; multiple of 8 (bf16) / 4 (fp32) */
  int64_t stride_head; /* elements; multiple of 8 (bf16) / 4 (fp32) */
} dbsa_tensor;

/*
 * Stage 1, many-shot encoding (Sec. 2.1): for every token i of the pool and every
 * query head h,  O[i,h,:] = sum_j softmax_j(scale * q[i,h,:].k[j,h/r,:]) v[j,h/r,:]
 * over the keys j the layout lists for i: the sink, the prev_window preceding
 * groups, and the own group up to and including i.  Sink rows attend the sink
 * causally.  r = n_q_heads / n_kv_heads (grouped-query attention, Sec. 4).
 *
 *   layout : a pre-encode layout with device lists.
 *   q, o   : [N, n_q_heads, D];  k, v : [N, n_kv_heads, D];  o is written.
 *   lse    : optional device float [n_q_heads][N]: natural-log softmax denominator.
 *   dtype  : DBSA_BF16 (MFMA kernel; fp32 accumulation, bf16 output; needs
 *            block_n == 64 and block_m in {32,64,128,256}) or DBSA_F32 (plain fp32
 *            kernel, any tile sizes).  head_dim in {64, 128}.
 * Errors: INVALID_ARG, UNSUPPORTED, HIP.
 */
int dbsa_preencode_attn(const dbsa_layout* layout, dbsa_tensor q, dbsa_tensor k, dbsa_tensor v, dbsa_tensor o,
                        float* lse, int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                        float softmax_scale, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Stage 2, query prefill (Sec. 2.2): token a of query u attends the sink, every
 * key of u's selected groups (read in place from the pool, no concatenation
 * copy), and its own tokens b <= a; one softmax over the union.
 *
 *   layout                 : a query-stage layout with device lists.
 *   q_self, o              : [sum T, n_q_heads, D], queries packed by cu_qlens.
 *   k_self, v_self         : [sum T, n_kv_heads, D].
 *   k_pool, v_pool         : [N, n_kv_heads, D].
 *   lse                    : optional device float [n_q_heads][sum T].
 *   workspace              : optional (NULL / 0): device memory, 16-byte aligned, of
 *                            dbsa_workspace_bytes(); see there.  A smaller one is ignored.
 * Same dtype / tile-size rules and errors as dbsa_preencode_attn.
 */
int dbsa_query_attn(const dbsa_layout* layout, dbsa_tensor q_self, dbsa_tensor k_self, dbsa_tensor v_self,
                    dbsa_tensor k_pool, dbsa_tensor v_pool, dbsa_tensor o, float* lse, int32_t dtype,
                    int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float softmax_scale, void* workspace,
                    size_t workspace_bytes, void* stream);

/*
 * Stage 2, one autoregressive step (Sec. 2.2): the new token of query u attends
 * the sink, u's selected groups and ALL of u's own cached keys [0, self_len[u]).
 * The caller appends the new token's K/V to the cache before the call and counts
 * it in self_len.  Runs a split-KV pass (one partial softmax state per split) and
 * a merge pass  m* = max m_s,  l* = sum l_s e^(m_s-m*),  o = sum acc_s e^(m_s-m*) / l*.
 *
 *   q_step, o               : [B, n_q_heads, D]  (stride_tok = stride between queries).
 *   k_selfcache, v_selfcache: [B, Tmax, n_kv_heads, D]; stride_tok/stride_head as
 *                             usual, stride_query elements between queries.
 *   self_len                : device int32 [B], 1 <= self_len[u] <= Tmax.
 *   workspace               : device memory of >= dbsa_workspace_bytes() bytes,
 *                             16-byte aligned; contents are overwritten.
 * Same dtype rules; block_n == 64 for DBSA_BF16.  Errors add WORKSPACE.
 *
 * Successive calls on one layout alternate the direction in which every run of keys is walked
 * (front to back, back to front): a step reads the same selected keys as the step before, more
 * of them than the last-level cache holds, and what the previous step read last is still there.
 * The two directions differ by fp32 summation order only.  Only a call that passes every check
 * and is launched changes the direction: a rejected call leaves the next one as it would have
 * been.  Calls on one layout from several threads are safe; they merely share that alternation.
 * The call only launches kernels (no allocation, no memset, no host wait), so it may be
 * recorded into a HIP graph by stream capture; the direction is fixed at capture time.
 */
int dbsa_decode_attn(const dbsa_layout* layout, dbsa_tensor q_step, dbsa_tensor k_selfcache, dbsa_tensor v_selfcache,
                     const int32_t* self_len, int64_t stride_query, dbsa_tensor k_pool, dbsa_tensor v_pool,
                     dbsa_tensor o, int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                     float softmax_scale, void* workspace, size_t workspace_bytes, void* stream);

/*
 * dbsa_decode_attn for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, arithmetic and results as dbsa_decode_attn, but the partial softmax states go
 * to a fixed buffer of DBSA_STATIC_SCRATCH_BYTES that is part of the library image (one copy
 * per GPU the library runs on, held until the process ends).  The call allocates nothing on
 * the device and frees nothing.
 * Limit: the step's partial states -- (head_dim + 4) floats per query head and slot, slots =
 * max(B * n_split, slot_ptr[B]) -- must fit the buffer, else DBSA_ERR_WORKSPACE and nothing
 * is launched (config 3 needs about 14 MiB).  Nothing in the buffer has to start at zero: every
 * slot a step reads was written by the same step.  All calls on one GPU share the buffer, so
 * two calls of this entry point that overlap on one GPU (different streams, or replays of
 * graphs that recorded it) race; calls on one stream are ordered and safe.
 */
#define DBSA_STATIC_SCRATCH_BYTES (32u << 20)
int dbsa_decode_attn_static(const dbsa_layout* layout, dbsa_tensor q_step, dbsa_tensor k_selfcache,
                            dbsa_tensor v_selfcache, const int32_t* self_len, int64_t stride_query, dbsa_tensor k_pool,
                            dbsa_tensor v_pool, dbsa_tensor o, int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads,
                            int32_t head_dim, float softmax_scale, void* stream);

/*
 * ---- query stage with re-positioning (Sec. 2.2) --------------------------------------------
 * The paper caches the pool's keys before the rotary transformation and, per test query,
 * re-applies it to the concatenated selected caches with new in-order position ids.  Here the
 * cached keys carry the rotation of the id they were ENCODED with instead (an invertible
 * change of what is stored), and a run of keys is moved to its new ids by rotating the query
 * row the opposite way -- rotary scores depend on id differences only.  One key tensor serves
 * every query, which is what lets decode fetch a group once for all queries that selected it.
 * Rotary convention: channel i pairs with channel i + D/2, angle = id * inv_freq[i].
 */

/*
 * table[n][i] = (cos, sin)(n * inv_freq[i]) as fp32 pairs, n < n_pos, i < head_dim/2, evaluated
 * in fp64 on the device.  inv_freq: host, [head_dim/2]; table: device, n_pos * head_dim floats,
 * 16-byte aligned.  Enqueued on `stream`.  Errors: INVALID_ARG, HIP.
 */
int dbsa_rope_table(const double* inv_freq, int32_t head_dim, int32_t n_pos, float* table, void* stream);

/*
 * out[t][h] = x[t][h] rotated at id positions[t] (device int32 [n_tokens]), or at first_id + t
 * when positions is NULL: the encoding-time rotation (pool keys: ids 0 .. N-1, Sec. 2.1; a
 * query's own keys: their index inside the query).  x and out may be the same tensor.  With
 * positions == NULL the ids are known to the host: INVALID_ARG unless 0 <= first_id and
 * first_id + n_tokens <= n_pos.  ids read from `positions` live on the device and are not checked:
 * the kernel clamps each to [0, n_pos), so an id outside the table gives the rotation of the
 * nearest table row instead of a fault; keeping them inside is the caller's duty.  head_dim a
 * multiple of 16 up to 128.  Errors: INVALID_ARG, UNSUPPORTED, HIP.
 */
int dbsa_rope_apply(dbsa_tensor x, dbsa_tensor out, int32_t n_tokens, int32_t n_heads, int32_t head_dim, int32_t dtype,
                    const int32_t* positions, int32_t first_id, const float* table, int32_t n_pos, void* stream);

/*
 * dbsa_query_attn with re-positioning.  q_self is UN-rotated; k_self holds each query's own keys
 * rotated at their index inside the query; k_pool holds pool keys rotated at their token index.
 * rope_table as written by dbsa_rope_table with n_pos > list_shift[e] + rows of the Q tile for
 * every list entry (else INVALID_ARG; 2 * pool tokens + the longest query always suffices: a
 * group that moves towards the front of the cache is reached by rotating the query FORWARD).  Same
 * dtypes and shapes as dbsa_query_attn: bf16 with head_dim 128 runs the pipelined matrix kernel, any
 * other shape the plain fp32-arithmetic one.  Everything else as dbsa_query_attn.
 */
int dbsa_query_attn_rope(const dbsa_layout* layout, dbsa_tensor q_self, dbsa_tensor k_self, dbsa_tensor v_self,
                         dbsa_tensor k_pool, dbsa_tensor v_pool, dbsa_tensor o, float* lse, const float* rope_table,
                         int32_t rope_n_pos, int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                         float softmax_scale, void* workspace, size_t workspace_bytes, void* stream);

/*
 * dbsa_decode_attn with re-positioning.  q_step is UN-rotated; the self caches hold keys rotated
 * at their index inside the query (the new token, index self_len[u] - 1, included).  A row looks
 * up id qref_shift[ref] + self_len[u] - 1.  self_len lives on the device, so the host bounds it by
 * what a query's cache can hold, Tmax = stride_query / k_selfcache.stride_tok tokens: INVALID_ARG
 * unless rope_n_pos > max(qref_shift) + Tmax - 1 (2 * pool tokens + Tmax always suffices).  A
 * self_len beyond Tmax is the caller's error; the kernel clamps the id to the table.
 * Same dtypes and shapes as dbsa_decode_attn: bf16 with head_dim 128 and 32 % (n_q_heads /
 * n_kv_heads) == 0 runs the group-major matrix kernel, any other shape the plain one.
 */
int dbsa_decode_attn_rope(const dbsa_layout* layout, dbsa_tensor q_step, dbsa_tensor k_selfcache,
                          dbsa_tensor v_selfcache, const int32_t* self_len, int64_t stride_query, dbsa_tensor k_pool,
                          dbsa_tensor v_pool, dbsa_tensor o, const float* rope_table, int32_t rope_n_pos,
                          int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                          float softmax_scale, void* workspace, size_t workspace_bytes, void* stream);

/*
 * dbsa_decode_attn over a pool whose keys and values are stored as 8-bit floats (Sec. 6 names
 * KV-cache quantisation as compatible with the method; the decode step is bound by the bytes
 * of the selected caches, Sec. 4).  k_pool8 / v_pool8: device bytes [N, n_kv_heads, D] in the
 * OCP e4m3 format (1-4-3, bias 7, no infinities), strides in bytes and multiples of 16;
 * the value of an element is byte * k_scale[kv head] (v_scale likewise), scales: device float
 * [n_kv_heads].  Quantising is the caller's business; the result is defined on the
 * de-quantised values.  q_step, the self caches (the query's own keys, never quantised) and o
 * are bf16.  head_dim 128, block_n 64, 32 % (n_q_heads / n_kv_heads) == 0 (else UNSUPPORTED).
 * Everything else (workspace, alternating walk direction, errors) as dbsa_decode_attn.
 */
int dbsa_decode_attn_kv8(const dbsa_layout* layout, dbsa_tensor q_step, dbsa_tensor k_selfcache,
                         dbsa_tensor v_selfcache, const int32_t* self_len, int64_t stride_query, dbsa_tensor k_pool8,
                         dbsa_tensor v_pool8, const float* k_scale, const float* v_scale, dbsa_tensor o,
                         int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float softmax_scale,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * dbsa_decode_attn_kv8 with re-positioning (Sec. 2.2), as dbsa_decode_attn_rope: q_step is
 * UN-rotated, the pool keys were rotated at their encoding ids BEFORE they were quantised, the
 * self caches hold bf16 keys rotated at their index inside the query; rope_table / rope_n_pos
 * as there.  Errors as both.
 */
int dbsa_decode_attn_kv8_rope(const dbsa_layout* layout, dbsa_tensor q_step, dbsa_tensor k_selfcache,
                              dbsa_tensor v_selfcache, const int32_t* self_len, int64_t stride_query,
                              dbsa_tensor k_pool8, dbsa_tensor v_pool8, const float* k_scale, const float* v_scale,
                              dbsa_tensor o, const float* rope_table, int32_t rope_n_pos, int32_t n_q_heads,
                              int32_t n_kv_heads, int32_t head_dim, float softmax_scale, void* workspace,
                              size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DBSA_H_ */
