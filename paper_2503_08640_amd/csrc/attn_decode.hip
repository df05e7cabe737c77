// Group-major split-KV decode for bf16, head_dim 128 on gfx950 (Sec. 2.2: one new token per
// query attends the sink, the query's selected groups and its own cached keys).
//
// Queries that selected the same group read the same keys, and a decode step is bound by
// HBM traffic, so the unit of work is not (query, split) but (run of KV tiles of one
// segment, up to 32 queries that use it): the run is fetched ONCE and scored against all of
// them on the matrix cores.  A workgroup is ONE wave that owns 32 score columns =
// (32 / r) queries x the r query heads of one KV head, and walks the run once per batch of
// 32 / r queries.  Every (item, query) pair writes one partial softmax state (m, l,
// unnormalised O) into its slot; a second kernel merges the slots of a query
// (m* = max m_s, l* = sum l_s 2^(m_s - m*), o = sum O_s 2^(m_s - m*) / l*).
//
// Tiles move as in the prefill kernel (global_load_lds_dwordx4 into XOR-swizzled LDS), in
// half tiles of 32 keys whose K and V parts are separate load groups, through a wave-private
// ring of three 8-KiB slots: no workgroup barrier; a slot is refilled as soon as the product
// that reads it is issued, so that 16 KiB per wave are in flight while it computes, and six
// single-wave workgroups per CU (24 KiB of LDS each) keep enough bytes outstanding to cover
// HBM latency.  What matters most for the speed of a step is that its workgroups fit the
// chip in ONE round: a half-filled second round costs a whole item time.
#include <atomic>
#include <cstdint>

#include "kernels.hpp"
#include "mfma_common.hpp"

namespace {

using namespace dbsa_mfma;

constexpr int kD = 128;
constexpr int kHalf = 32;                      // keys per half tile
constexpr int kRowBytes = kD * 2;              // 256
constexpr int kHalfBytes = kHalf * kRowBytes;  // 8 KiB per K or V half tile
constexpr int kSlots = 3;                      // ring slots of one K or V half tile each
constexpr int kLdsBytes = kSlots * kHalfBytes;  // 24 KiB per wave: six waves per CU
constexpr int kLoadsPerGroup = kHalfBytes / 1024;  // LDS-DMA instructions per K or V half tile
constexpr float kRescaleSlack = 8.f;

// What one workgroup of the group-major step walks: a run of consecutive pool keys for up to 32
// queries, or one query's own cache.
struct DecodeItem {
  int hk;         // KV head
  int batch;      // query batch of the launch row
  int item;       // pool items first, then one self item per query
  bool self_item;
  int n_q, first_key, n_keys, self_u;
};

// Workgroup id -> (KV head, launch row, item in the row's block of 8), the item fastest.  A row
// is (block, query batch); the rows of one block follow each other, so the workgroups that walk
// one item's keys for different query batches have ids 8 apart: they start together AND on the
// same XCD (ids are dealt to the 8 XCDs in turn), and all but the first find the keys in that
// XCD's L2.  Rows exist only for batches some item of the block has.  False: the id names no item.
// Everything the first loads need (the run, the query references) is one load away from the item
// index: all workgroups of a step start together, and every further dependent load at their start
// is a microsecond or two in which no tile data moves.  (The schedule lists are read-only while a
// kernel runs: scalar loads through the constant path.)
__device__ DBSA_INLINE bool locate_decode_item(const AttnParams& p, DecodeItem& it) {
  const int in_block = blockIdx.x % 8;
  const int row_id = (blockIdx.x / 8) % p.launch_rows;
  it.hk = (blockIdx.x / 8) / p.launch_rows;
  const int row = ((const_words)(reinterpret_cast<uintptr_t>(p.gm_rows)))[p.row_offset + row_id];
  it.batch = row & 0xFF;
  const int block = row >> 8;
  it.self_item = block >= p.n_pool_blocks;
  it.item = it.self_item ? p.n_gm_items + 8 * (block - p.n_pool_blocks) + in_block : 8 * block + in_block;
  if (it.item >= (it.self_item ? p.n_gm_items + p.n_queries : p.n_gm_items)) return false;
  const const_words runs = (const_words)(reinterpret_cast<uintptr_t>(p.gm_item_run));
  it.n_q = 1, it.first_key = 0, it.n_keys = 0, it.self_u = 0;
  if (!it.self_item) {
    it.first_key = runs[4 * it.item + 0];
    it.n_keys = runs[4 * it.item + 1];
    it.n_q = runs[4 * it.item + 2];
  } else {
    it.self_u = it.item - p.n_gm_items;
    it.n_keys = __builtin_amdgcn_readfirstlane(p.self_len[it.self_u]);
  }
  return true;
}

// A lane's score column: lanes l and l + 32 share column l % 32 = (query l32 / r of the wave's
// batch, head l32 % r of the KV head).
struct DecodeColumn {
  int slot, head;
  bool valid;        // the batch has a query for this column (the others compute on a repeated reference)
  const __bf16* qp;  // the query row, at this lane's first channel
  const float* rot;  // ROPE: table row of the column, 16 floats (cos, sin of 8 channel pairs) per (chunk c < 4, half)
};

// pass: the wave's query batch (of 32 / r queries) inside the item; active: the wave has a batch.
// ROPE: the row is rotated at the id that stands for the new in-order position of the item's keys
// (Sec. 2.2): shift of the reference + the query's own length - 1.
// (The addresses are formed here, before the tile loads go out: they wait for the query reference
// just loaded, and that wait must not include the tile loads.)
template <bool ROPE>
__device__ DBSA_INLINE DecodeColumn decode_column(const AttnParams& p, const DecodeItem& it, int pass, bool active, int r,
                                                  int l32, int half) {
  DecodeColumn c;
  const int q_local = pass * (32 / r) + l32 / r;  // index into the item's query list (< 32 also without a batch)
  c.valid = active && q_local < it.n_q;
  int u = it.self_u, rot_id = 0;
  if (it.self_item) {
    c.slot = static_cast<int>(p.gm_slot_ptr[it.self_u + 1]) - 1;
  } else {
    // (query, slot, shift, 0); references past the item's last one repeat it
    typedef int intx4 __attribute__((ext_vector_type(4)));
    const intx4 ref = *reinterpret_cast<const intx4*>(p.gm_ref_pad + (static_cast<int64_t>(it.item) * 32 + q_local) * 4);
    u = ref[0];
    c.slot = ref[1];
    if (ROPE) rot_id = ref[2];
  }
  c.head = it.hk * r + l32 % r;
  c.rot = nullptr;
  if (ROPE) {
    rot_id = min(max(rot_id + p.self_len[u] - 1, 0), p.rope_n_pos - 1);
    c.rot = p.rope_table + static_cast<int64_t>(rot_id) * kD + 16 * half;
    asm volatile("" : "+v"(c.rot));
  }
  c.qp = static_cast<const __bf16*>(p.q.ptr) + static_cast<int64_t>(u) * p.q.stride_tok +
         static_cast<int64_t>(c.head) * p.q.stride_head + 8 * half;
  asm volatile("" : "+v"(c.qp));
  return c;
}

// The pieces of one half tile (32 keys) against the 32 columns of a wave.  The kernels differ in
// where K and V come from and in what they issue between the pieces; the arithmetic is shared.
union ProbFrag {
  bf16x8 v[2];
  bf16x2 p2[8];
};

// scores of a bf16 K half tile in LDS (swizzled as the loads of decode_group_kernel leave it):
// two accumulator chains of four MFMAs instead of one of eight, half the latency
__device__ DBSA_INLINE floatx16 half_tile_scores(const lds_byte* ks, int k_base, const bf16x8 (&qf)[kD / 16]) {
  floatx16 s, s2;
#pragma unroll
  for (int i = 0; i < 16; ++i) s[i] = 0.f, s2[i] = 0.f;
#pragma unroll
  for (int c = 0; c < kD / 16; c += 2) {
    const bf16x8 a = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(ks + (k_base ^ (32 * c)));
    const bf16x8 a2 = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(ks + (k_base ^ (32 * (c + 1))));
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[c], s, 0, 0, 0);
    s2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a2, qf[c + 1], s2, 0, 0, 0);
  }
  s += s2;
  return s;
}

// masks the keys past `len`, moves the lazily rescaled running state (o, m_run, l_run) and leaves
// the probabilities as the B operand of the second product
__device__ DBSA_INLINE void half_tile_softmax(floatx16& s, int len, int half, floatx16 (&o)[kD / 32], float& m_run,
                                              float& l_run, ProbFrag& pf) {
  if (len < kHalf) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key_local = 8 * (i / 4) + 4 * half + (i % 4);
      s[i] = key_local < len ? s[i] : -INFINITY;
    }
  }
  float mx = s[0];
#pragma unroll
  for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[i]);
  mx = half_swap_max(mx);
  if (__builtin_amdgcn_ballot_w64(mx > m_run + kRescaleSlack) != 0) {
    const float m_new = fmaxf(m_run, mx);
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    l_run *= alpha;
#pragma unroll
    for (int ob = 0; ob < kD / 32; ++ob) o[ob] *= alpha;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float p0 = __builtin_amdgcn_exp2f(s[2 * i] - m_run);
    const float p1 = __builtin_amdgcn_exp2f(s[2 * i + 1] - m_run);
    pf.p2[i] = __builtin_convertvector(floatx2{p0, p1}, bf16x2);
    l_run += p0 + p1;
  }
}

// o += V^T P^T for a bf16 V half tile in LDS (transposed fragments through the LDS transpose read)
__device__ DBSA_INLINE void half_tile_weigh(const lds_byte* vs, int v_base, const ProbFrag& pf, floatx16 (&o)[kD / 32]) {
#pragma unroll
  for (int ch = 0; ch < 2; ++ch)
#pragma unroll
    for (int ob = 0; ob < kD / 32; ++ob) {
      const lds_byte* vp = vs + (v_base ^ (64 * ob)) + 16 * ch * kRowBytes;
      const bf16x4 lo = lds_read_tr(vp);
      const bf16x4 hi = lds_read_tr(vp + 8 * kRowBytes);
      const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      o[ob] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf.v[ch], o[ob], 0, 0, 0);
    }
}

// One whole half tile: ks / vs are the K and V half tiles in LDS, len the valid keys, k_base /
// v_base this lane's fragment offsets; the running state is updated in place.
__device__ DBSA_INLINE void half_tile_attend(const lds_byte* ks, const lds_byte* vs, int len, int k_base, int v_base, int half,
                                             const bf16x8 (&qf)[kD / 16], floatx16 (&o)[kD / 32], float& m_run,
                                             float& l_run) {
  floatx16 s = half_tile_scores(ks, k_base, qf);
  ProbFrag pf;
  half_tile_softmax(s, len, half, o, m_run, l_run, pf);
  half_tile_weigh(vs, v_base, pf, o);
}

// The partial softmax state of a valid column: accumulators (times out_scale), running maximum, row sum.
__device__ DBSA_INLINE void store_partial_state(const AttnParams& p, const DecodeColumn& c, int half, const floatx16 (&o)[kD / 32],
                                                float m_run, float l_run, float out_scale) {
  const float l_tot = half_swap_sum(l_run);
  if (!c.valid) return;
  float* part = p.partial + (static_cast<int64_t>(c.slot) * p.n_q_heads + c.head) * (kD + kPartialPad);
#pragma unroll
  for (int ob = 0; ob < kD / 32; ++ob)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      *reinterpret_cast<floatx4*>(part + 32 * ob + 8 * g + 4 * half) =
          floatx4{o[ob][4 * g] * out_scale, o[ob][4 * g + 1] * out_scale, o[ob][4 * g + 2] * out_scale,
                  o[ob][4 * g + 3] * out_scale};
  if (half == 0) {
    part[kD] = m_run;
    part[kD + 1] = l_tot;
  }
}

// ROPE: the query row is un-rotated and is rotated here at the id that stands for the new
// in-order position of the item's keys (Sec. 2.2), see AttnParams::gm_ref_pad.
template <bool ROPE>
__global__ __launch_bounds__(64, 2) void decode_group_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  lds_byte* lds = (lds_byte*)smem;
  const int lane = threadIdx.x, l32 = lane % 32, half = lane / 32;
  const int r = p.n_q_heads / p.n_kv_heads;
  const int qpw = 32 / r;  // queries per wave
  // ---- the item: a run of pool tiles for several queries, or one query's own cache ----
  DecodeItem it;
  if (!locate_decode_item(p, it)) return;
  const int hk = it.hk, pass = it.batch, n_q = it.n_q, first_key = it.first_key, n_keys = it.n_keys, self_u = it.self_u;
  const bool self_item = it.self_item;
  // the run is a stretch of consecutive key rows: first_key .. first_key + n_keys
  const int n_half = (n_keys + kHalf - 1) / kHalf;
  const __bf16* kbase = self_item ? static_cast<const __bf16*>(p.k_self.ptr) + self_u * p.stride_query +
                                        hk * p.k_self.stride_head
                                  : static_cast<const __bf16*>(p.k_pool.ptr) + hk * p.k_pool.stride_head;
  const __bf16* vbase = self_item ? static_cast<const __bf16*>(p.v_self.ptr) + self_u * p.stride_query +
                                        hk * p.v_self.stride_head
                                  : static_cast<const __bf16*>(p.v_pool.ptr) + hk * p.v_pool.stride_head;
  const int k_stride = static_cast<int>(self_item ? p.k_self.stride_tok : p.k_pool.stride_tok);
  const int v_stride = static_cast<int>(self_item ? p.v_self.stride_tok : p.v_pool.stride_tok);

  // half tile hh -> (first token, number of valid keys)
  // (walked from the far end when p.decode_reverse is set, see there)
  auto half_ref = [&](int hh, int& start, int& len) {
    const int pos = p.decode_reverse ? n_half - 1 - hh : hh;
    start = first_key + pos * kHalf;
    len = min(kHalf, n_keys - pos * kHalf);
  };

  // ---- loads: 8 K blocks and 8 V blocks of 1 KiB per half tile ----
  // block b holds rows 4b .. 4b+3; lane -> row 4b + lane/16, slot lane%16 (swizzled).  For a
  // full half tile the per-lane byte offset only depends on b % 4 (K) or not on b at all (V);
  // the 4b rows go into the uniform base pointer.
  unsigned k_lane_off[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
    k_lane_off[j] = static_cast<unsigned>((lane / 16) * k_stride + (((lane % 16) ^ (4 * j + lane / 16)) * 8)) * 2u;
  const unsigned v_lane_off =
      static_cast<unsigned>((lane / 16) * v_stride + (((lane % 16) ^ (4 * ((lane / 16) % 4))) * 8)) * 2u;
  // K and V of a half tile are separate load groups of kLoadsPerGroup instructions each, so that a
  // slot can be refilled as soon as ITS product has consumed it
  auto issue_k = [&](int hh) {
    int start, len;
    half_ref(hh, start, len);
    lds_byte* stage = lds + ((2 * hh) % kSlots) * kHalfBytes;
    const __bf16* kb = kbase + static_cast<int64_t>(start) * k_stride;
    if (len == kHalf) {
#pragma unroll
      for (int b = 0; b < kLoadsPerGroup; ++b)
        dma16(kb + static_cast<int64_t>(4 * b) * k_stride, k_lane_off[b % 4], stage + b * 1024);
    } else {
#pragma unroll
      for (int b = 0; b < kLoadsPerGroup; ++b) {
        const int row_in = 4 * b + lane / 16;
        const int row = min(row_in, len - 1);  // rows past the tail repeat the last key
        dma16(kb, static_cast<unsigned>(row * k_stride + (((lane % 16) ^ (row_in % 16)) * 8)) * 2u,
              stage + b * 1024);
      }
    }
  };
  auto issue_v = [&](int hh) {
    int start, len;
    half_ref(hh, start, len);
    lds_byte* stage = lds + ((2 * hh + 1) % kSlots) * kHalfBytes;
    const __bf16* vb = vbase + static_cast<int64_t>(start) * v_stride;
    if (len == kHalf) {
#pragma unroll
      for (int b = 0; b < kLoadsPerGroup; ++b)
        dma16(vb + static_cast<int64_t>(4 * b) * v_stride, v_lane_off, stage + b * 1024);
    } else {
#pragma unroll
      for (int b = 0; b < kLoadsPerGroup; ++b) {
        const int row_in = 4 * b + lane / 16;
        const int row = min(row_in, len - 1);
        dma16(vb, static_cast<unsigned>(row * v_stride + (((lane % 16) ^ (4 * (row_in % 4))) * 8)) * 2u,
              stage + b * 1024);
      }
    }
  };
  // wait until at most `groups` load groups (0..2) are still outstanding
  auto wait_groups = [&](int groups) {
    if (groups >= 2) wait_vmcnt<2 * kLoadsPerGroup>();
    else if (groups == 1) wait_vmcnt<kLoadsPerGroup>();
    else wait_vmcnt<0>();
  };

  const int k_base = l32 * kRowBytes + ((half ^ (l32 % 16)) * 16);
  const int v_base = (4 * half + (lane % 16) / 4) * kRowBytes +
                     (((2 * (l32 / 16) + (lane % 4) / 2) ^ (4 * ((lane % 16) / 4))) * 16) + (lane % 2) * 8;
  const float c2 = p.scale_log2e;
  const int n_pass = (n_q + qpw - 1) / qpw;

  // One workgroup per batch of 32 / r queries of the item: an item that serves more queries than
  // one wave has columns is walked by several workgroups side by side instead of by one workgroup
  // several times, which would make it the last to finish.
  if (pass >= n_pass) return;
  {
    // ---- this lane's column: query and head ----
    const DecodeColumn col = decode_column<ROPE>(p, it, pass, true, r, l32, half);

    // ---- wave-private ring of three 8-KiB slots: load groups go out in the order K(0) V(0) K(1)
    // V(1) K(2) ..., group g into slot g % 3, and group g+3 as soon as the product that reads group
    // g is issued: two slots are in flight while the third is being computed on.  The first
    // groups are requested before the query row, so that both latencies run together. ----
    issue_k(0);
    issue_v(0);
    if (1 < n_half) issue_k(1);
    bf16x8 qf[kD / 16];
    load_query_fragments<ROPE>(col.qp, col.rot, c2, qf);
    floatx16 o[kD / 32];
#pragma unroll
    for (int ob = 0; ob < kD / 32; ++ob)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[ob][i] = 0.f;
    float m_run = -1.0e30f, l_run = 0.f;

    for (int hh = 0; hh < n_half; ++hh) {
      // K(hh) has landed once only the groups issued after it are outstanding: V(hh), K(hh+1)
      wait_groups(1 + (hh + 1 < n_half ? 1 : 0));
      int start, len;
      half_ref(hh, start, len);
      const lds_byte* ks = lds + ((2 * hh) % kSlots) * kHalfBytes;
      const lds_byte* vs = lds + ((2 * hh + 1) % kSlots) * kHalfBytes;

      floatx16 s = half_tile_scores(ks, k_base, qf);
      // the K slot is free (its LDS reads were consumed by the MFMAs above): it takes the group
      // three places on, V(hh+1)
      if (hh + 1 < n_half) issue_v(hh + 1);
      ProbFrag pf;
      half_tile_softmax(s, len, half, o, m_run, l_run, pf);
      // V(hh) has landed once only K(hh+1) and V(hh+1) are outstanding
      wait_groups(hh + 1 < n_half ? 2 : 0);
      half_tile_weigh(vs, v_base, pf, o);
      if (hh + 2 < n_half) issue_k(hh + 2);  // into the slot V(hh) just left
    }

    store_partial_state(p, col, half, o, m_run, l_run, 1.f);
  }
}

// ---------------------------------------------------------------------------------------------
// The same walk for layouts whose items serve MORE queries than one wave has columns (many
// concurrent queries, high retrieval ratios): the W waves of a workgroup take W consecutive query
// batches of one item and share every half tile in LDS, so the keys travel from L2 to LDS once
// per W batches instead of once per batch.  Each wave issues 1/W of a tile's load instructions
// and waits for its own; ONE barrier per half tile then makes the tile visible to all waves and
// tells that every wave is done with the tile before, whose slot takes the loads of the tile two
// places on.  Ring of three (K, V) pairs of half tiles: two pairs in flight while one is used.
constexpr int kPairs = 3;
constexpr int kPairBytes = 2 * kHalfBytes;       // 16 KiB
constexpr int kLdsShared = kPairs * kPairBytes;  // 48 KiB per workgroup: three workgroups per CU

template <int W, bool ROPE>
__global__ __launch_bounds__(64 * W) void decode_group_shared_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  lds_byte* lds = (lds_byte*)smem;
  constexpr int kPerWave = kLoadsPerGroup / W;  // load instructions per wave per K or V half tile
  static_assert(kLoadsPerGroup % W == 0, "waves share the load instructions evenly");
  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) / 64);
  const int lane = threadIdx.x % 64, l32 = lane % 32, half = lane / 32;
  const int r = p.n_q_heads / p.n_kv_heads;
  const int qpw = 32 / r;  // queries per wave
  // a row's batch counts batches of W * qpw queries here
  DecodeItem it;
  if (!locate_decode_item(p, it)) return;
  const int hk = it.hk, wg_batch = it.batch, n_q = it.n_q, first_key = it.first_key, n_keys = it.n_keys, self_u = it.self_u;
  const bool self_item = it.self_item;
  const int n_half = (n_keys + kHalf - 1) / kHalf;
  const int n_pass = (n_q + qpw - 1) / qpw;
  // (everything up to here is the same for all waves: the workgroup leaves as one)
  if (wg_batch * W >= n_pass) return;
  const int pass = wg_batch * W + wave;
  const bool active = pass < n_pass;  // a wave without a batch still loads its share and keeps the barriers

  const __bf16* kbase = self_item ? static_cast<const __bf16*>(p.k_self.ptr) + self_u * p.stride_query +
                                        hk * p.k_self.stride_head
                                  : static_cast<const __bf16*>(p.k_pool.ptr) + hk * p.k_pool.stride_head;
  const __bf16* vbase = self_item ? static_cast<const __bf16*>(p.v_self.ptr) + self_u * p.stride_query +
                                        hk * p.v_self.stride_head
                                  : static_cast<const __bf16*>(p.v_pool.ptr) + hk * p.v_pool.stride_head;
  const int k_stride = static_cast<int>(self_item ? p.k_self.stride_tok : p.k_pool.stride_tok);
  const int v_stride = static_cast<int>(self_item ? p.v_self.stride_tok : p.v_pool.stride_tok);
  auto half_ref = [&](int hh, int& start, int& len) {
    const int pos = p.decode_reverse ? n_half - 1 - hh : hh;
    start = first_key + pos * kHalf;
    len = min(kHalf, n_keys - pos * kHalf);
  };

  // this wave's load instructions of a half tile are the 1-KiB blocks b = wave + W * j (rows
  // 4b .. 4b+3; lane -> row 4b + lane/16, 16-byte slot lane%16, swizzled as in decode_group_kernel)
  unsigned k_lane_off[kPerWave];
#pragma unroll
  for (int j = 0; j < kPerWave; ++j)
    k_lane_off[j] = static_cast<unsigned>((lane / 16) * k_stride +
                                          (((lane % 16) ^ (4 * ((wave + W * j) % 4) + lane / 16)) * 8)) * 2u;
  const unsigned v_lane_off =
      static_cast<unsigned>((lane / 16) * v_stride + (((lane % 16) ^ (4 * ((lane / 16) % 4))) * 8)) * 2u;
  auto issue_pair = [&](int hh) {
    int start, len;
    half_ref(hh, start, len);
    lds_byte* k_stage = lds + (hh % kPairs) * kPairBytes;
    lds_byte* v_stage = k_stage + kHalfBytes;
    const __bf16* kb = kbase + static_cast<int64_t>(start) * k_stride;
    const __bf16* vb = vbase + static_cast<int64_t>(start) * v_stride;
    if (len == kHalf) {
#pragma unroll
      for (int j = 0; j < kPerWave; ++j) {
        const int b = wave + W * j;
        dma16(kb + static_cast<int64_t>(4 * b) * k_stride, k_lane_off[j], k_stage + b * 1024);
      }
#pragma unroll
      for (int j = 0; j < kPerWave; ++j) {
        const int b = wave + W * j;
        dma16(vb + static_cast<int64_t>(4 * b) * v_stride, v_lane_off, v_stage + b * 1024);
      }
    } else {
#pragma unroll
      for (int j = 0; j < kPerWave; ++j) {
        const int b = wave + W * j;
        const int row_in = 4 * b + lane / 16;
        const int row_k = min(row_in, len - 1);  // rows past the tail repeat the last key
        dma16(kb, static_cast<unsigned>(row_k * k_stride + (((lane % 16) ^ (row_in % 16)) * 8)) * 2u,
              k_stage + b * 1024);
      }
#pragma unroll
      for (int j = 0; j < kPerWave; ++j) {
        const int b = wave + W * j;
        const int row_in = 4 * b + lane / 16;
        const int row_v = min(row_in, len - 1);
        dma16(vb, static_cast<unsigned>(row_v * v_stride + (((lane % 16) ^ (4 * (row_in % 4))) * 8)) * 2u,
              v_stage + b * 1024);
      }
    }
  };

  const int k_base = l32 * kRowBytes + ((half ^ (l32 % 16)) * 16);
  const int v_base = (4 * half + (lane % 16) / 4) * kRowBytes +
                     (((2 * (l32 / 16) + (lane % 4) / 2) ^ (4 * ((lane % 16) / 4))) * 16) + (lane % 2) * 8;
  const float c2 = p.scale_log2e;

  // ---- this lane's column: query and head ----
  const DecodeColumn col = decode_column<ROPE>(p, it, pass, active, r, l32, half);

  issue_pair(0);
  if (1 < n_half) issue_pair(1);
  bf16x8 qf[kD / 16];
  load_query_fragments<ROPE>(col.qp, col.rot, c2, qf);
  floatx16 o[kD / 32];
#pragma unroll
  for (int ob = 0; ob < kD / 32; ++ob)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[ob][i] = 0.f;
  float m_run = -1.0e30f, l_run = 0.f;

  for (int hh = 0; hh < n_half; ++hh) {
    // this wave's part of pair hh has landed once only its part of pair hh+1 is outstanding
    if (hh + 1 < n_half) wait_vmcnt<2 * kPerWave>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");  // no LDS read of this pair may move above the barrier
    // every wave is past pair hh-1: its slot takes pair hh+2
    if (hh + 2 < n_half) issue_pair(hh + 2);
    if (!active) continue;
    int start, len;
    half_ref(hh, start, len);
    const lds_byte* ks = lds + (hh % kPairs) * kPairBytes;
    const lds_byte* vs = ks + kHalfBytes;

    half_tile_attend(ks, vs, len, k_base, v_base, half, qf, o, m_run, l_run);
  }

  store_partial_state(p, col, half, o, m_run, l_run, 1.f);
}

// ---------------------------------------------------------------------------------------------
// Pool items over an fp8 (e4m3) pool: half the bytes per key.  Same work decomposition as
// decode_group_kernel (one wave per (item, KV head, query batch)).  A half tile of 32 keys
// arrives as 4 KiB of K bytes and 4 KiB of V bytes in a ring of four 4-KiB slots (K(h), V(h),
// K(h+1), V(h+1)).  K fragments are read from the staged bytes directly and widened to bf16 in
// registers; V is widened into one bf16 working tile (the transposed fragment reads need 16-bit
// elements), same swizzle as the bf16 kernel.  24 KiB of LDS per wave keeps six waves per CU.
// The per-head scales ride on Q (keys) and on the partial accumulators (values), so no key or
// value is ever multiplied.
constexpr int kSlot8 = 4096;
constexpr int kLds8 = 4 * kSlot8 + kHalfBytes;  // 24 KiB per wave
constexpr int kLoads8 = 4;                      // load instructions per group (the K or the V bytes of a half tile)

__device__ inline bf16x8 widen8(unsigned w0, unsigned w1) {
  union {
    bf16x8 v;
    bf16x2 p2[4];
  } out;
  out.p2[0] = __builtin_convertvector(__builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(w0), false), bf16x2);
  out.p2[1] = __builtin_convertvector(__builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(w0), true), bf16x2);
  out.p2[2] = __builtin_convertvector(__builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(w1), false), bf16x2);
  out.p2[3] = __builtin_convertvector(__builtin_amdgcn_cvt_pk_f32_fp8(static_cast<int>(w1), true), bf16x2);
  return out.v;
}

template <bool ROPE>
__global__ __launch_bounds__(64, 2) void decode_group_kv8_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  lds_byte* lds = (lds_byte*)smem;
  lds_byte* work_v = lds + 4 * kSlot8;
  const int lane = threadIdx.x, l32 = lane % 32, half = lane / 32;
  const int r = p.n_q_heads / p.n_kv_heads;
  const int qpw = 32 / r;
  // this launch covers the rows of pool items only
  DecodeItem it;
  if (!locate_decode_item(p, it) || it.self_item) return;
  const int hk = it.hk, pass = it.batch, n_q = it.n_q, first_key = it.first_key, n_keys = it.n_keys;
  const int n_half = (n_keys + kHalf - 1) / kHalf;
  if (pass >= (n_q + qpw - 1) / qpw) return;

  const unsigned char* kbase = static_cast<const unsigned char*>(p.k_pool.ptr) + hk * p.k_pool.stride_head;
  const unsigned char* vbase = static_cast<const unsigned char*>(p.v_pool.ptr) + hk * p.v_pool.stride_head;
  const int k_stride = static_cast<int>(p.k_pool.stride_tok), v_stride = static_cast<int>(p.v_pool.stride_tok);
  auto half_ref = [&](int hh, int& start, int& len) {
    const int pos = p.decode_reverse ? n_half - 1 - hh : hh;
    start = first_key + pos * kHalf;
    len = min(kHalf, n_keys - pos * kHalf);
  };
  // Load instruction j fills rows 8j .. 8j+7 of a staged operand (128-byte rows; lane -> row
  // 8j + lane/8, 16-byte slot lane%8); rows past the tail repeat the last key.  K slots are
  // swizzled by row % 8 (= lane/8) for the 64-bit fragment reads: 32 rows x one 8-byte piece
  // would otherwise sit 16 deep on the same banks.
  auto issue_k = [&](int hh) {
    int start, len;
    half_ref(hh, start, len);
    lds_byte* stage = lds + ((2 * hh) % 4) * kSlot8;
    const unsigned char* kb = kbase + static_cast<int64_t>(start) * k_stride;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = min(8 * j + lane / 8, len - 1);
      dma16(kb, static_cast<unsigned>(row * k_stride + (((lane % 8) ^ (lane / 8)) * 16)), stage + j * 1024);
    }
  };
  auto issue_v = [&](int hh) {
    int start, len;
    half_ref(hh, start, len);
    lds_byte* stage = lds + ((2 * hh + 1) % 4) * kSlot8;
    const unsigned char* vb = vbase + static_cast<int64_t>(start) * v_stride;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = min(8 * j + lane / 8, len - 1);
      dma16(vb, static_cast<unsigned>(row * v_stride + (lane % 8) * 16), stage + j * 1024);
    }
  };
  auto wait_groups = [&](int groups) {  // at most `groups` load groups (0..3) still in flight
    if (groups >= 3) wait_vmcnt<3 * kLoads8>();
    else if (groups == 2) wait_vmcnt<2 * kLoads8>();
    else if (groups == 1) wait_vmcnt<kLoads8>();
    else wait_vmcnt<0>();
  };

  // K fragment c of key row l32: channels 16c + 8*half .. +7 = 8 bytes of slot c ^ (l32 % 8)
  const int k8_base = l32 * 128 + 8 * half;
  const int k8_swz = l32 % 8;
  const int v_base = (4 * half + (lane % 16) / 4) * kRowBytes +
                     (((2 * (l32 / 16) + (lane % 4) / 2) ^ (4 * ((lane % 16) / 4))) * 16) + (lane % 2) * 8;

  // ---- this lane's column (ROPE as in decode_group_kernel: the stored keys keep their encoding-time rotation) ----
  const DecodeColumn col = decode_column<ROPE>(p, it, pass, true, r, l32, half);
  issue_k(0);
  issue_v(0);
  if (1 < n_half) {
    issue_k(1);
    issue_v(1);
  }
  const float c2 = p.scale_log2e * p.k_scale8[hk];
  const float v_scale = p.v_scale8[hk];
  bf16x8 qf[kD / 16];
  load_query_fragments<ROPE>(col.qp, col.rot, c2, qf);
  floatx16 o[kD / 32];
#pragma unroll
  for (int ob = 0; ob < kD / 32; ++ob)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[ob][i] = 0.f;
  float m_run = -1.0e30f, l_run = 0.f;

  for (int hh = 0; hh < n_half; ++hh) {
    const bool more = hh + 1 < n_half;
    // K(hh) has landed once only the groups issued after it are outstanding: V(hh), K(hh+1), V(hh+1)
    wait_groups(more ? 3 : 1);
    int start, len;
    half_ref(hh, start, len);
    const lds_byte* ks = lds + ((2 * hh) % 4) * kSlot8;
    const lds_byte* vs = lds + ((2 * hh + 1) % 4) * kSlot8;

    floatx16 s, s2;
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f, s2[i] = 0.f;
#pragma unroll
    for (int c = 0; c < kD / 16; c += 2) {
      typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
      const uintx2 w = *reinterpret_cast<const __attribute__((address_space(3))) uintx2*>(ks + k8_base + ((c ^ k8_swz) * 16));
      const uintx2 w2 =
          *reinterpret_cast<const __attribute__((address_space(3))) uintx2*>(ks + k8_base + (((c + 1) ^ k8_swz) * 16));
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(widen8(w[0], w[1]), qf[c], s, 0, 0, 0);
      s2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(widen8(w2[0], w2[1]), qf[c + 1], s2, 0, 0, 0);
    }
    s += s2;
    // the K slot is free (its bytes are in registers): it takes the K bytes two half tiles on
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (hh + 2 < n_half) issue_k(hh + 2);
    ProbFrag pf;
    half_tile_softmax(s, len, half, o, m_run, l_run, pf);
    // V(hh) has landed once only K(hh+1), V(hh+1) and K(hh+2) are outstanding
    wait_groups((more ? 2 : 0) + (hh + 2 < n_half ? 1 : 0));
    // staged V bytes -> the swizzled bf16 working tile
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
      typedef __attribute__((address_space(3))) bf16x8* tile_ptr;
      const int row = 8 * j + lane / 8, s0 = 2 * (lane % 8);
      const uintx4 vx = *reinterpret_cast<const __attribute__((address_space(3))) uintx4*>(vs + j * 1024 + lane * 16);
      *(tile_ptr)(work_v + row * kRowBytes + ((s0 ^ (4 * (row % 4))) * 16)) = widen8(vx[0], vx[1]);
      *(tile_ptr)(work_v + row * kRowBytes + (((s0 + 1) ^ (4 * (row % 4))) * 16)) = widen8(vx[2], vx[3]);
    }
    // the V slot is free: it takes the V bytes two half tiles on
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (hh + 2 < n_half) issue_v(hh + 2);
    half_tile_weigh(work_v, v_base, pf, o);
    // the working tile is rewritten in the next round: its reads must have returned
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }

  store_partial_state(p, col, half, o, m_run, l_run, v_scale);
}

// ---------------------------------------------------------------------------------------------
// fp8 pool, many queries per item: the W waves of a workgroup take W query batches of one item
// (as in decode_group_shared_kernel) and share not only the staged bytes but their WIDENING: a
// half tile's 4 KiB of K bytes and 4 KiB of V bytes arrive in a ring of three staging pairs; each
// wave widens the rows it fetched itself (1/W of the pair: 32 bytes -> 32 bf16 per lane) into ONE
// bf16 working pair laid out exactly as the bf16 kernels' tiles, and all waves run the bf16
// arithmetic on that pair.  Two barriers per half tile: before the widening (every wave is done
// with the working pair of the half tile before) and after it (the working pair is complete).
constexpr int kStagePair8 = 2 * kSlot8;                               // 8 KiB of bytes per (K, V) half tile
constexpr int kLdsShared8 = kPairs * kStagePair8 + kPairBytes;        // 24 KiB staging + 16 KiB working pair

template <int W, bool ROPE>
__global__ __launch_bounds__(64 * W) void decode_group_kv8_shared_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  lds_byte* lds = (lds_byte*)smem;
  lds_byte* work_k = lds + kPairs * kStagePair8;
  lds_byte* work_v = work_k + kHalfBytes;
  static_assert(kLoads8 % W == 0, "waves share the load instructions evenly");
  constexpr int kPerWave = kLoads8 / W;  // load instructions per wave per K or V half tile (8 rows each)
  const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) / 64);
  const int lane = threadIdx.x % 64, l32 = lane % 32, half = lane / 32;
  const int r = p.n_q_heads / p.n_kv_heads;
  const int qpw = 32 / r;
  // this launch covers the rows of pool items only; a row's batch counts batches of W * qpw queries
  DecodeItem it;
  if (!locate_decode_item(p, it) || it.self_item) return;
  const int hk = it.hk, wg_batch = it.batch, n_q = it.n_q, first_key = it.first_key, n_keys = it.n_keys;
  const int n_half = (n_keys + kHalf - 1) / kHalf;
  const int n_pass = (n_q + qpw - 1) / qpw;
  if (wg_batch * W >= n_pass) return;  // (the same for all waves: the workgroup leaves as one)
  const int pass = wg_batch * W + wave;
  const bool active = pass < n_pass;

  const unsigned char* kbase = static_cast<const unsigned char*>(p.k_pool.ptr) + hk * p.k_pool.stride_head;
  const unsigned char* vbase = static_cast<const unsigned char*>(p.v_pool.ptr) + hk * p.v_pool.stride_head;
  const int k_stride = static_cast<int>(p.k_pool.stride_tok), v_stride = static_cast<int>(p.v_pool.stride_tok);
  auto half_ref = [&](int hh, int& start, int& len) {
    const int pos = p.decode_reverse ? n_half - 1 - hh : hh;
    start = first_key + pos * kHalf;
    len = min(kHalf, n_keys - pos * kHalf);
  };
  // load instruction j of a staged operand fills rows 8j .. 8j+7 (128-byte rows; lane -> row
  // 8j + lane/8, 16 bytes lane%8; rows past the tail repeat the last key); wave w issues the
  // instructions j = w + W*i and later widens exactly those rows
  auto issue_pair = [&](int hh) {
    int start, len;
    half_ref(hh, start, len);
    lds_byte* k_stage = lds + (hh % kPairs) * kStagePair8;
    lds_byte* v_stage = k_stage + kSlot8;
    const unsigned char* kb = kbase + static_cast<int64_t>(start) * k_stride;
    const unsigned char* vb = vbase + static_cast<int64_t>(start) * v_stride;
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      const int j = wave + W * i;
      const int row_k = min(8 * j + lane / 8, len - 1);
      dma16(kb, static_cast<unsigned>(row_k * k_stride + (lane % 8) * 16), k_stage + j * 1024);
    }
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      const int j = wave + W * i;
      const int row_v = min(8 * j + lane / 8, len - 1);
      dma16(vb, static_cast<unsigned>(row_v * v_stride + (lane % 8) * 16), v_stage + j * 1024);
    }
  };
  // this wave's rows of staged pair hh -> bf16 working pair: lane -> row 8j + lane/8, channels
  // 16*(lane%8) .. +15 = the 16-byte slots 2*(lane%8) and 2*(lane%8)+1 of the 256-byte bf16 row,
  // K slots swizzled by row % 16, V slots by 4*(row % 4) (the bf16 kernels' layouts)
  auto widen_pair = [&](int hh) {
    const lds_byte* k_stage = lds + (hh % kPairs) * kStagePair8;
    const lds_byte* v_stage = k_stage + kSlot8;
    typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
    typedef const __attribute__((address_space(3))) uintx4* bytes_ptr;
    typedef __attribute__((address_space(3))) bf16x8* tile_ptr;
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      const int j = wave + W * i;
      const int row = 8 * j + lane / 8, s0 = 2 * (lane % 8);
      const uintx4 kx = *(bytes_ptr)(k_stage + j * 1024 + lane * 16);
      const uintx4 vx = *(bytes_ptr)(v_stage + j * 1024 + lane * 16);
      *(tile_ptr)(work_k + row * kRowBytes + ((s0 ^ (row % 16)) * 16)) = widen8(kx[0], kx[1]);
      *(tile_ptr)(work_k + row * kRowBytes + (((s0 + 1) ^ (row % 16)) * 16)) = widen8(kx[2], kx[3]);
      *(tile_ptr)(work_v + row * kRowBytes + ((s0 ^ (4 * (row % 4))) * 16)) = widen8(vx[0], vx[1]);
      *(tile_ptr)(work_v + row * kRowBytes + (((s0 + 1) ^ (4 * (row % 4))) * 16)) = widen8(vx[2], vx[3]);
    }
  };

  const int k_base = l32 * kRowBytes + ((half ^ (l32 % 16)) * 16);
  const int v_base = (4 * half + (lane % 16) / 4) * kRowBytes +
                     (((2 * (l32 / 16) + (lane % 4) / 2) ^ (4 * ((lane % 16) / 4))) * 16) + (lane % 2) * 8;

  // ---- this lane's column ----
  const DecodeColumn col = decode_column<ROPE>(p, it, pass, active, r, l32, half);
  issue_pair(0);
  if (1 < n_half) issue_pair(1);
  const float c2 = p.scale_log2e * p.k_scale8[hk];
  const float v_scale = p.v_scale8[hk];
  bf16x8 qf[kD / 16];
  load_query_fragments<ROPE>(col.qp, col.rot, c2, qf);
  floatx16 o[kD / 32];
#pragma unroll
  for (int ob = 0; ob < kD / 32; ++ob)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[ob][i] = 0.f;
  float m_run = -1.0e30f, l_run = 0.f;

  for (int hh = 0; hh < n_half; ++hh) {
    // this wave's bytes of pair hh have landed once only its part of pair hh+1 is outstanding
    if (hh + 1 < n_half) wait_vmcnt<2 * kPerWave>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();  // every wave is done with the working pair of half tile hh-1 ...
    asm volatile("" ::: "memory");
    // ... and widened its rows of staged pair hh-1 before that: the slot takes pair hh+2
    if (hh + 2 < n_half) issue_pair(hh + 2);
    widen_pair(hh);
    __syncthreads();  // the working pair is complete (LDS writes of all waves visible)
    if (!active) continue;
    int start, len;
    half_ref(hh, start, len);
    half_tile_attend(work_k, work_v, len, k_base, v_base, half, qf, o, m_run, l_run);
  }

  store_partial_state(p, col, half, o, m_run, l_run, v_scale);
}

// Merge the partial states of one (query, head): slots [slot_ptr[u], slot_ptr[u+1]).
// 2 x 128 threads: thread (part, d) owns output channel d for the slots of its parity.  The
// per-slot maxima and sums are read with one slot per thread (not one after the other by
// everyone), the weights 2^(m_s - m*) go through LDS, and the weighted sum of the accumulators
// runs with eight independent loads in flight per thread; the two parities meet in LDS.
constexpr int kMergeThreads = 2 * kD;
__global__ __launch_bounds__(kMergeThreads) void decode_group_merge_kernel(AttnParams p) {
  constexpr int kRow = kD + kPartialPad, kCap = 256, kWaves = kMergeThreads / 64;
  __shared__ float w_sh[kCap];
  __shared__ float red[2][kWaves];
  __shared__ float acc_sh[kD];
  const int u = blockIdx.x / p.n_q_heads, head = blockIdx.x % p.n_q_heads;
  const int t = threadIdx.x, d = t % kD, part = t / kD;
  const int s0 = static_cast<int>(p.gm_slot_ptr[u]), s1 = static_cast<int>(p.gm_slot_ptr[u + 1]);
  const float* partial = p.partial + static_cast<int64_t>(head) * kRow;
  const int64_t slot_stride = static_cast<int64_t>(p.n_q_heads) * kRow;

  auto block_reduce = [&](float x, bool is_max, int which) {
    for (int o = 32; o > 0; o >>= 1) {
      const float y = __shfl_xor(x, o, 64);
      x = is_max ? fmaxf(x, y) : x + y;
    }
    if (t % 64 == 0) red[which][t / 64] = x;
    __syncthreads();
    float r = red[which][0];
    for (int w = 1; w < kWaves; ++w) r = is_max ? fmaxf(r, red[which][w]) : r + red[which][w];
    return r;
  };

  float m = -1.0e30f;
  for (int s = s0 + t; s < s1; s += kMergeThreads) m = fmaxf(m, partial[s * slot_stride + kD]);
  const float m_star = block_reduce(m, true, 0);

  float l = 0.f, acc = 0.f;
  for (int base = s0; base < s1; base += kCap) {
    const int n = min(kCap, s1 - base);
    __syncthreads();  // previous round's weights are consumed
    for (int i = t; i < n; i += kMergeThreads) {
      const float w = __builtin_amdgcn_exp2f(partial[(base + i) * slot_stride + kD] - m_star);
      w_sh[i] = w;
      l = fmaf(partial[(base + i) * slot_stride + kD + 1], w, l);
    }
    __syncthreads();
    const float* col = partial + static_cast<int64_t>(base) * slot_stride + d;
    int i = part;
    for (; i + 14 < n; i += 16) {
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = col[(i + 2 * j) * slot_stride];
#pragma unroll
      for (int j = 0; j < 8; ++j) acc = fmaf(v[j], w_sh[i + 2 * j], acc);
    }
    for (; i < n; i += 2) acc = fmaf(col[i * slot_stride], w_sh[i], acc);
  }
  const float l_star = block_reduce(l, false, 1);
  if (part == 1) acc_sh[d] = acc;
  __syncthreads();
  if (part == 0) {
    __bf16* o = static_cast<__bf16*>(const_cast<void*>(p.o.ptr));
    o[static_cast<int64_t>(u) * p.o.stride_tok + static_cast<int64_t>(head) * p.o.stride_head + d] =
        static_cast<__bf16>((acc + acc_sh[d]) / l_star);
  }
}

}  // namespace

namespace {
// one workgroup per (KV head, launch row, item of the row's block)
dim3 decode_grid(const AttnParams& p) { return dim3(static_cast<unsigned>(p.n_kv_heads) * p.launch_rows * 8); }
}  // namespace

namespace {
template <int W>
hipError_t launch_shared8(const AttnParams& p, hipStream_t stream) {
  static std::atomic<bool> attr_set{false};  // setting it twice from two threads is harmless
  if (!attr_set) {
    for (const void* f : {reinterpret_cast<const void*>(decode_group_kv8_shared_kernel<W, false>),
                          reinterpret_cast<const void*>(decode_group_kv8_shared_kernel<W, true>)}) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsShared8);
      if (e != hipSuccess) return e;
    }
    attr_set = true;
  }
  const dim3 grid = decode_grid(p), block(64 * W);
  if (p.rope_table)
    decode_group_kv8_shared_kernel<W, true><<<grid, block, kLdsShared8, stream>>>(p);
  else
    decode_group_kv8_shared_kernel<W, false><<<grid, block, kLdsShared8, stream>>>(p);
  return hipGetLastError();
}
}  // namespace

// p.decode_waves as for launch_decode_group (pool rows; the self rows below are single batches)
hipError_t launch_decode_group_kv8(const AttnParams& p_in, hipStream_t stream) {
  static std::atomic<bool> attr_set{false};  // setting it twice from two threads is harmless
  if (!attr_set) {
    for (const void* f : {reinterpret_cast<const void*>(decode_group_kv8_kernel<false>),
                          reinterpret_cast<const void*>(decode_group_kv8_kernel<true>)}) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kLds8);
      if (e != hipSuccess) return e;
    }
    for (const void* f : {reinterpret_cast<const void*>(decode_group_kernel<false>),
                          reinterpret_cast<const void*>(decode_group_kernel<true>)}) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
      if (e != hipSuccess) return e;
    }
    attr_set = true;
  }
  AttnParams p = p_in;
  if (p.n_gm_items > 0) {
    p.row_offset = 0;
    p.launch_rows = p.gm_pool_rows;
    hipError_t e;
    if (p.decode_waves == 4)
      e = launch_shared8<4>(p, stream);
    else if (p.decode_waves == 2)
      e = launch_shared8<2>(p, stream);
    else {
      if (p.rope_table)
        decode_group_kv8_kernel<true><<<decode_grid(p), dim3(64), kLds8, stream>>>(p);
      else
        decode_group_kv8_kernel<false><<<decode_grid(p), dim3(64), kLds8, stream>>>(p);
      e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
  }
  // every query's own (bf16) cache: the self items of the ordinary kernel
  p.row_offset = p.gm_pool_rows;
  p.launch_rows = p.gm_n_rows - p.gm_pool_rows;
  if (p.rope_table)
    decode_group_kernel<true><<<decode_grid(p), dim3(64), kLdsBytes, stream>>>(p);
  else
    decode_group_kernel<false><<<decode_grid(p), dim3(64), kLdsBytes, stream>>>(p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  decode_group_merge_kernel<<<dim3(p.n_queries * p.n_q_heads), dim3(kMergeThreads), 0, stream>>>(p);
  return hipGetLastError();
}

namespace {
template <int W>
hipError_t launch_shared(const AttnParams& p, hipStream_t stream) {
  static std::atomic<bool> attr_set{false};  // setting it twice from two threads is harmless
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_group_shared_kernel<W, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsShared);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_group_shared_kernel<W, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kLdsShared);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const dim3 grid = decode_grid(p), block(64 * W);
  if (p.rope_table)
    decode_group_shared_kernel<W, true><<<grid, block, kLdsShared, stream>>>(p);
  else
    decode_group_shared_kernel<W, false><<<grid, block, kLdsShared, stream>>>(p);
  return hipGetLastError();
}
}  // namespace

// p.decode_waves = waves per workgroup (1, 2 or 4; the launch rows in p are those of batches of
// decode_waves * 32 / r queries)
hipError_t launch_decode_group(const AttnParams& p_in, hipStream_t stream) {
  AttnParams p = p_in;
  static std::atomic<bool> attr_set{false};  // setting it twice from two threads is harmless
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_group_kernel<false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(decode_group_kernel<true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipError_t e;
  if (p.decode_matrix) {
    // Many queries per group: the pool items as a contraction (64 query rows per wave, four query heads
    // of a KV head as the four waves of a workgroup, see attn_prefill64.hip), every query's own cache
    // in the single-wave kernel, then the same merge.  The partial states land in the same slots.
    AttnParams g = p;
    g.sched_rec = p.mx_sched_rec;
    g.sched_ptr = p.mx_sched_ptr;
    g.sched_classes = p.mx_classes;
    g.n_head_blocks = p.n_q_heads / 4;
    g.list_ent = p.mx_ent;
    g.heads_per_block = 4;
    g.block_m = 64;
    g.query_stage = 0;
    g.q_split = 1;
    g.lse = nullptr;
    e = launch_decode_matrix_items(g, stream);
    if (e != hipSuccess) return e;
    p.row_offset = p.gm_pool_rows;
    p.launch_rows = p.gm_n_rows - p.gm_pool_rows;
    if (p.rope_table)
      decode_group_kernel<true><<<decode_grid(p), dim3(64), kLdsBytes, stream>>>(p);
    else
      decode_group_kernel<false><<<decode_grid(p), dim3(64), kLdsBytes, stream>>>(p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    decode_group_merge_kernel<<<dim3(p.n_queries * p.n_q_heads), dim3(kMergeThreads), 0, stream>>>(p);
    return hipGetLastError();
  }
  p.row_offset = 0;
  p.launch_rows = p.gm_n_rows;
  if (p.decode_waves == 4) {
    e = launch_shared<4>(p, stream);
  } else if (p.decode_waves == 2) {
    e = launch_shared<2>(p, stream);
  } else {
    const dim3 grid = decode_grid(p), block(64);
    if (p.rope_table)
      decode_group_kernel<true><<<grid, block, kLdsBytes, stream>>>(p);
    else
      decode_group_kernel<false><<<grid, block, kLdsBytes, stream>>>(p);
    e = hipGetLastError();
  }
  if (e != hipSuccess) return e;
  decode_group_merge_kernel<<<dim3(p.n_queries * p.n_q_heads), dim3(kMergeThreads), 0, stream>>>(p);
  return hipGetLastError();
}
