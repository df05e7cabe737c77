// Launch parameters shared by api.hip and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

// A partial softmax state of one (slot, query head) is head_dim accumulator floats, the
// running max, the row sum and two floats of padding (rows stay 16-byte aligned).
constexpr int kPartialPad = 4;

struct TensorView {
  const void* ptr;
  int64_t stride_tok;   // elements
  int64_t stride_head;  // elements
};

// One description covers the three attention calls.  Prefill-shaped calls
// (pre-encode, query) walk list_ent through list_ptr per Q tile; the decode call
// walks dec_ent through split_ptr per (query, split) and then the query's own cache.
struct AttnParams {
  // lists (device)
  const int32_t* qtile_tab;  // [n_qtiles][4]
  const int64_t* list_ptr;   // [n_qtiles+1]
  const int32_t* list_ent;   // [n_ent][2]
  const int32_t* order;      // [n_qtiles]
  const int32_t* dec_ent;    // [n_dec_ent][2]
  const int64_t* split_ptr;  // [B][n_split+1]
  const int64_t* gm_slot_ptr;  // [B+1]
  int32_t n_gm_items;
  int32_t gm_max_queries;      // most queries any group-major item serves
  int32_t n_qtiles, n_split, n_queries;
  // tensors
  TensorView q, o;            // rows: tokens (prefill) or queries (decode)
  TensorView k_pool, v_pool;  // [N, Hkv, D]
  TensorView k_self, v_self;  // prefill: [sum T, Hkv, D]; decode: cache of one query, + stride_query per query
  int64_t stride_query;       // decode only (elements)
  const int32_t* self_len;    // decode only, device [B]
  float* lse;                 // optional [Hq][n_rows]
  int64_t lse_stride;         // rows per head in lse
  float* partial;             // decode: [slot][Hq][D + kPartialPad]; per-query splits use slot = u*n_split + s;
                              // split prefill: [row][Hq][q_split][D + kPartialPad]
  // group-major decode launch: workgroup id -> row (id / 8) % launch_rows of gm_rows + row_offset,
  // KV head (id / 8) / launch_rows, item 8 * block + id % 8 of the row's block; blocks below
  // n_pool_blocks hold pool items, the others self items (one per query)
  const int32_t* gm_rows;     // (block << 8 | query batch), pool rows first
  int32_t gm_n_rows, gm_pool_rows;
  int32_t n_pool_blocks;
  int32_t row_offset, launch_rows;
  const float* k_scale8;      // decode over an fp8 pool: k = k8 * k_scale8[kv head], v = v8 * v_scale8[kv head]
  const float* v_scale8;
  int32_t decode_reverse;     // decode: walk every run of keys from its last half tile to its first
  int32_t decode_waves;       // decode: waves per workgroup that share an item's tiles (1, 2 or 4)
  int32_t q_split;            // prefill: runs each Q tile's list is cut into (1 = no split, no merge pass)
  int32_t n_rows;             // prefill: rows of q / o
  // shapes
  int32_t n_q_heads, n_kv_heads, block_m, block_n;
  int32_t heads_per_block;    // query heads handled by one workgroup (divides Hq/Hkv)
  // persistent prefill-shaped launch (null: one workgroup per Q tile): workgroup w serves head block
  // w % n_head_blocks and records sched_ptr[c] .. sched_ptr[c+1]-1, c = w / n_head_blocks, of
  // sched_rec = [n_qtiles][4] (q_start, q_len, first list entry, entries)
  const int32_t* sched_rec;
  const int32_t* sched_ptr;
  int32_t sched_classes, n_head_blocks;
  // rows gathered through references (launch_decode_matrix_items): [n_refs][2] = (row of q, partial slot)
  const int32_t* gather_refs;
  const int32_t* gather_shift;  // [n_refs]: with re-positioning, rotation id of reference i's row = gather_shift[i] + self_len - 1
  // decode step: 1 = the pool items run as a contraction through launch_decode_matrix_items with the
  // schedule mx_sched_* over list entries mx_ent, the self items in the ordinary kernel (gm_rows then
  // holds the table of single-wave workgroups)
  int32_t decode_matrix;
  const int32_t* mx_sched_rec;
  const int32_t* mx_sched_ptr;
  const int32_t* mx_ent;
  int32_t mx_classes;
  int32_t query_stage;        // prefill-shaped calls: 1 = query prefill (lists may name self tiles), 0 = pre-encode
  // re-positioning (null table: inputs carry their final positions already)
  const float* rope_table;    // [rope_n_pos][D/2][2] fp32 (cos, sin) of id * inv_freq
  int32_t rope_n_pos;
  const int32_t* list_shift;  // [n_ent]: rotation id of row i of a Q tile for entry e = list_shift[e] + i
  const int32_t* dec_shift;   // [n_dec_ent]: rotation id of a decode row for dec_ent entry e = dec_shift[e] + self_len - 1
  const int32_t* gm_item_run; // group-major decode: [n_gm_items][4] = (first key row, keys, queries, 0)
  const int32_t* gm_ref_pad;  // [n_gm_items][32][4] = (query, slot, shift, 0), tail repeats the last reference;
                              // rotation id of a decode row = shift + self_len - 1
  float scale;                // softmax scale
  float scale_log2e;          // scale * log2(e)
};

// bf16 MFMA kernels (attn_mfma.hip)
hipError_t launch_prefill_mfma(const AttnParams& p, int head_dim, hipStream_t stream);
// software-pipelined variant for head_dim 128 (attn_prefill.hip)
hipError_t launch_prefill_pipelined(const AttnParams& p, hipStream_t stream);
// the same mathematics with 64 query rows per wave, one wave per SIMD (attn_prefill64.hip); kernel
// only: launch_prefill_pipelined runs the merge pass of a split launch
hipError_t launch_prefill64(const AttnParams& p, hipStream_t stream);
// the same kernel over rows gathered through references, leaving partial softmax states: the pool
// items of a decode step with many queries per group (attn_prefill64.hip)
hipError_t launch_decode_matrix_items(const AttnParams& p, hipStream_t stream);
// group-major split-KV decode + merge for head_dim 128 (attn_decode.hip)
hipError_t launch_decode_group(const AttnParams& p, hipStream_t stream);
// the same with pool K/V stored as fp8 (e4m3) bytes and per-KV-head scales
hipError_t launch_decode_group_kv8(const AttnParams& p, hipStream_t stream);
hipError_t launch_decode_mfma(const AttnParams& p, int head_dim, hipStream_t stream);
hipError_t launch_decode_merge(const AttnParams& p, int head_dim, bool out_bf16, hipStream_t stream);

// rotary tables and the encoding-time rotation (rope.hip)
hipError_t launch_rope_table(const double* inv_freq, int head_dim, int n_pos, float* table, hipStream_t stream);
hipError_t launch_rope_apply(const TensorView& x, const TensorView& out, int n_tokens, int n_heads, int head_dim,
                             bool bf16, const int32_t* positions, int first_id, const float* table, int n_pos,
                             hipStream_t stream);

// plain fp32-arithmetic kernels for fp32 or bf16 storage (attn_plain.hip)
hipError_t launch_prefill_plain(const AttnParams& p, int head_dim, bool bf16_storage, hipStream_t stream);
hipError_t launch_decode_plain(const AttnParams& p, int head_dim, bool bf16_storage, hipStream_t stream);
