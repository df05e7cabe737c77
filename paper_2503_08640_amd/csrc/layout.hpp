// Internal definition of the opaque dbsa_layout object: host index lists built by
// layout.cpp and their device mirrors filled in by api.hip.
#pragma once

#include <atomic>
#include <cstdint>
#include <mutex>
#include <vector>

#include "../../include/dbsa.h"

struct dbsa_device_lists {
  void* base = nullptr;           // one allocation holds every list below
  void* staging = nullptr;        // pinned host buffer the lists were copied from
  size_t capacity = 0;            // bytes of base / staging
  int device = -1;
  int32_t* qtile_tab = nullptr;   // [n_qtiles][4]
  int64_t* list_ptr = nullptr;    // [n_qtiles+1]
  int32_t* list_ent = nullptr;    // [n_ent][2]
  int32_t* order = nullptr;       // [n_qtiles]
  int32_t* dec_ent = nullptr;     // [n_dec_ent][2]
  int64_t* split_ptr = nullptr;   // [B][n_split+1]
  int64_t* gm_slot_ptr = nullptr; // [B+1]
  int32_t* list_shift = nullptr;  // [n_ent]
  int32_t* dec_shift = nullptr;   // [n_dec_ent]
  int32_t* gm_qshift = nullptr;   // [n_qrefs]
  int32_t* mx_qrefs = nullptr;    // [n_mx_qrefs][2]
  int32_t* mx_qshift = nullptr;   // [n_mx_qrefs]
  int64_t* mx_slot_ptr = nullptr; // [B+1]
  int32_t* gm_item_run = nullptr; // [n_items][4]
  int32_t* gm_ref_pad = nullptr;  // [n_items][32][4]
  int32_t* gm_rows = nullptr;
  // room for ONE persistent-launch schedule (dbsa_layout::sched), filled by the first prefill-shaped
  // call that uses one
  int32_t* sched_rec = nullptr;   // [n_qtiles][4]
  int32_t* sched_ptr = nullptr;   // [kMaxSchedClasses + 1]
  void* sched_uploaded = nullptr; // event recorded behind the schedule's copy
  void* sched_stream = nullptr;   // stream of that copy
  // decode steps that run their pool items as a contraction (dbsa_layout::mx_rec): the segments'
  // tile entries, the flat references, and room for that launch's schedule, filled by the first
  // decode call that uses it
  int32_t* gm_seg_ent = nullptr;   // [n_seg_ent][2]
  int32_t* gm_qrefs = nullptr;     // [n_qrefs][2]
  int32_t* mx_sched_rec = nullptr; // [n_mx][4]
  int32_t* mx_sched_ptr = nullptr; // [kMaxSchedClasses + 1]
  void* mx_uploaded = nullptr;
  void* mx_stream = nullptr;
  // ordering of the asynchronous upload against the calls that read the lists (HIP handles kept
  // as plain pointers so that host-only code can include this header)
  void* upload_stream = nullptr;  // stream the lists were copied on
  void* uploaded = nullptr;       // event recorded behind that copy
};

struct dbsa_layout {
  bool query_stage = false;
  bool on_device = false;
  int32_t block_m = 0, block_n = 0;
  int32_t sink_len = 0, n_tokens = 0, n_groups = 0, prev_window = 0;
  int32_t n_queries = 0, n_query_tokens = 0, n_split = 0;

  std::vector<int32_t> qtile_tab;   // 4 per tile
  std::vector<int64_t> list_ptr;
  std::vector<int32_t> list_ent;    // 2 per entry
  std::vector<int32_t> order;
  std::vector<int64_t> dec_ptr;     // [B+1]
  std::vector<int32_t> dec_ent;     // 2 per entry
  std::vector<int64_t> split_ptr;   // [B][n_split+1]
  // group-major decode schedule: every KV chunk is walked once for all queries that use it
  int32_t gm_chunk_tiles = 0;
  std::vector<int64_t> gm_seg_ptr;  // [n_groups+2] offsets of the sink's and each group's tiles in gm_seg_ent
  std::vector<int32_t> gm_seg_ent;  // 2 per tile
  std::vector<int32_t> gm_items;    // 4 per item: (ent_begin, ent_count, qref_begin, n_q)
  std::vector<int32_t> gm_qrefs;    // 2 per reference: (query, slot)
  std::vector<int64_t> gm_slot_ptr; // [B+1]; the last slot of a query is its own-cache partial
  // re-positioning (Sec. 2.2: new in-order position ids for the concatenated selected caches).
  // Keys are stored rotated at the id they were encoded with (pool keys: their token index; a
  // query's own keys: their index inside the query), so moving a run of keys to its new ids is
  // the same as rotating the QUERY row back by the run's displacement.  A row with local index a
  // (inside its query) scores the keys of list entry e after a rotation at id  list_shift[e] +
  // (a - first local index of its Q tile);  a decode row of query u scores the keys of a
  // schedule item after a rotation at id  gm_qshift[ref] + self_len[u] - 1.
  std::vector<int32_t> list_shift;  // [n_ent]
  // the same for the per-query decode lists: the new token of a query whose cache holds n tokens (itself
  // included) scores the keys of dec_ent entry e after a rotation at id dec_shift[e] + n - 1
  std::vector<int32_t> dec_shift;   // [n_dec_ent]
  std::vector<int32_t> gm_qshift;   // [n_qrefs]
  std::vector<int32_t> cache_len;   // [B]: |D'| of query u = sink + its selected groups
  // what the decode kernel reads, flattened so that nothing it needs first hangs off another load:
  // per item (first key row, keys, queries, 0) and 32 references (query, slot, shift, 0), the
  // tail repeating the last real reference
  std::vector<int32_t> gm_item_run; // [n_items][4]
  std::vector<int32_t> gm_ref_pad;  // [n_items][32][4]
  // launch rows of the decode kernel, one table per number of queries a wave takes (32 >> k,
  // k = 0..5): a row is (block of 8 work items) << 8 | query batch, listed only where some item of
  // the block has that many queries; blocks of pool items first, then blocks of self items
  std::vector<int32_t> gm_rows;
  int32_t gm_rows_off[7] = {0, 0, 0, 0, 0, 0, 0};   // table k is gm_rows[off[k] .. off[k+1])
  int32_t gm_pool_rows[6] = {0, 0, 0, 0, 0, 0};     // rows of table k that belong to pool items
  float gm_walks_per_key[6] = {1, 1, 1, 1, 1, 1};   // batches per pool item at 32 >> k queries per wave, weighted by keys
  // Records for steps that run as a contraction (64 query rows per wave): [n_mx][4] = (first reference,
  // references (at most 64), first tile entry in gm_seg_ent, entries).  mx_row_fill: share of the 64 rows
  // that carry a query, weighted by tiles.
  // Layouts that fill kMatrixRowFill of the rows cut these records' runs to measure for mx_plan_workers
  // workers per KV head (compute units / 8): worker c of such a step takes records mx_plan_ptr[c] ..
  // mx_plan_ptr[c+1]-1 (mx_plan_ptr.size() - 1 workers carry records), and the records have references
  // and partial-state slots of their own (mx_qrefs = (query, slot), mx_qshift, mx_slot_ptr as gm_*; the
  // work items keep their runs of one length for every other kernel).  Other layouts: mx_plan_ptr empty,
  // the records are the work items' runs taken in pairs and refer to gm_qrefs.
  std::vector<int32_t> mx_rec;
  float mx_row_fill = 0.f;
  std::vector<int32_t> mx_plan_ptr;
  int32_t mx_plan_workers = 0;
  std::vector<int32_t> mx_qrefs, mx_qshift;
  std::vector<int64_t> mx_slot_ptr;
  // figures the attention calls need on every launch, taken once at build time
  int32_t gm_max_queries = 1;       // most queries any schedule item serves
  int64_t shortest_list = 0;        // fewest entries any Q tile lists
  int64_t max_rotation_id = -1;     // largest id a prefill row looks up: max(list_shift[e] + rows of the tile) - 1
  int64_t max_decode_shift = 0;     // largest gm_qshift: a decode row of self_len n looks up id shift + n - 1
  // compute units of the device the launches are sized for (set before the host lists are built;
  // 256 when the layout is built without a device)
  int32_t compute_units = 256;

  // Schedule of a persistent prefill-shaped launch for n_classes workers (dbsa_balance_schedule),
  // computed by the first call that needs one and kept: class c walks records
  // sched_ptr[c] .. sched_ptr[c+1]-1 of sched_rec, four words each (q_start, q_len, first list
  // entry, entries).  0 classes: none yet.
  mutable std::mutex sched_mutex;
  mutable int32_t sched_classes = 0;
  mutable std::vector<int32_t> sched_ptr, sched_rec;
  mutable bool sched_on_device = false;
  // the same for the records of mx_rec (a second, independent schedule)
  mutable int32_t mx_classes = 0;
  mutable std::vector<int32_t> mx_sched_ptr, mx_sched_rec;
  mutable bool mx_on_device = false;

  mutable dbsa_device_lists dev;
  // direction of the last walk over the pool's keys by an attention call on this layout (the
  // decode call alternates it); not part of the lists, hence mutable
  mutable std::atomic<int> last_walk_reversed{0};
  // streams that attention calls have read the device lists on; the block that holds the lists
  // is handed to another layout only when all of them have passed the point of the destroy call
  mutable std::mutex use_mutex;
  mutable std::vector<void*> used_streams;

  int64_t n_qtiles() const { return static_cast<int64_t>(qtile_tab.size() / 4); }
  int64_t n_ent() const { return static_cast<int64_t>(list_ent.size() / 2); }
};

constexpr int32_t kMaxSchedClasses = 512;
// share of a wave's 64 rows that must carry a query before a decode step runs its pool items as a
// contraction (measured on a 90k-token pool, 8 KV heads, 32-256 queries, with the runs cut to measure:
// at 0.24-0.5 the step is 3-26 % faster than with 32-column work items, at 0.18 and below 10-20 % slower)
constexpr float kMatrixRowFill = 0.22f;

// Deals the Q tiles of a layout to n_classes workers for a launch in which every worker walks its
// tiles one after the other: tiles are taken in launch order (owner-major, so that at any time all
// workers read the K/V of the same owner) in rounds of n_classes, and within a round the longest
// list goes to the worker with the least work so far.  Work of a tile = its list entries + a fixed
// cost per tile.  Pure host integer work.
void dbsa_balance_schedule(const dbsa_layout* L, int32_t n_classes, std::vector<int32_t>* class_ptr,
                           std::vector<int32_t>* rec);
// The dealing rule itself, over records of four words in launch order whose last word is the
// number of list entries.
void dbsa_balance_records(const std::vector<int32_t>& rec_in, int32_t n_classes, std::vector<int32_t>* class_ptr,
                          std::vector<int32_t>* rec);

// Pure host integer work; returns a DBSA_* code and fills `L` on success.
// first_group < 0: every segment; >= 0 (pre-encode only): Q tiles of groups first_group.. alone
int dbsa_build_host_lists(const dbsa_pool_desc* pool, const dbsa_select_desc* sel, int32_t first_group, int32_t block_m, int32_t block_n,
                          dbsa_layout* L);
