// bf16 MFMA attention for prefill-shaped calls (pre-encode, Sec. 2.1; query prefill, Sec. 2.2)
// at head_dim 128 on gfx950, with 64 query rows per wavefront and ONE wavefront per SIMD.
//
// Same mathematics, operand layouts and LDS swizzles as attn_prefill.hip (transposed scores
// S^T = K Q^T, per-lane softmax statistics, O^T = V^T P^T, tiles moved by
// global_load_lds_dwordx4).  What differs is the split of the work:
//
//   * a wave owns TWO blocks of 32 query rows (two tokens ranges of one head, or the same tokens
//     of two heads that share the KV head), so that every K or V fragment read from LDS feeds two
//     matrix instructions.  Its 128 output accumulators live in the accumulation registers; the
//     wave has the SIMD to itself (512 registers), and latencies are hidden by the order of the
//     instructions inside the wave, not by a second wave.
//   * the unit of the software pipeline is a HALF tile (32 keys), in three stages one step apart:
//       step h:   S(h+1) = K(h+1) Q^T     (16 matrix instructions)
//                 P(h)   = exp2(S(h))     (vector ALU, spread over the step)
//                 O     += V(h-1) P(h-1)  (16 matrix instructions)
//     No instruction of a step waits for a result of the same step: the matrix pipe runs 32
//     instructions back to back while the vector ALU turns the scores of the previous step into
//     the probabilities of the next one.
//   * one workgroup barrier per 64-key tile (two steps) publishes the tiles the LDS-DMA brought in.
//
// The running maximum of a row is set from the first half tile in which the row sees a key (a
// row starts in the state "no key seen", so a run of tiles may begin with tiles that are masked
// for some rows) and is then left alone: it only has to keep the probabilities inside what bf16
// and fp32 hold.  No row maxima are computed in the tile loop; the sum of a step's probabilities,
// which the row sum needs anyway, shows when a row has outgrown its maximum, and that step's
// probabilities are then made again around the true maximum before the product uses them
// (shifts are whole log2 units).
#include <atomic>
#include <cstdint>

#include "kernels.hpp"
#include "mfma_common.hpp"

namespace {
using namespace dbsa_mfma;

constexpr int kD = 128;
constexpr int kBN = 64;                       // keys per KV tile
constexpr int kRowBytes = kD * 2;             // 256
constexpr int kTileBytes = kBN * kRowBytes;   // 16 KiB per K or V tile
// Operand fragments are read from LDS kDist fragments (two matrix instructions each) before their use, into
// slot (index in the step) % kRing of a ring; kRing divides the fragments of every step, so that the fragments
// one step reads for the next land where that step looks for them.
constexpr int kRing = 8;
constexpr int kDist = 5;
// a lane's sum of the 16 probabilities of one step above which the step is redone around the true
// row maximum: below it every probability is under 2^10, far inside bf16 and fp32
constexpr float kOverflowSum = 1024.f;
constexpr float kNoKey = -3.0e38f;            // below every finite score: "this row has seen no key yet"

struct TileRef {
  int start, len;
  bool causal, self;
};

typedef int intx4 __attribute__((ext_vector_type(4)));

// Score products S = K Q^T as inline assembly, so that their operand classes are fixed by hand:
// the accumulators in ordinary vector registers (the vector ALU reads them next), the Q^T
// fragments in accumulation registers (they are matrix operands only), while the compiler keeps
// the output accumulators of the second product, which it sees as builtins, in accumulation
// registers.  Left to itself it puts every matrix result of a one-wave-per-SIMD kernel into
// accumulation registers and copies each score back before the exponential.
// The compiler does not know what these statements are, so the spacing rules between a matrix
// instruction and other users of its registers are kept by the order of the code: a score block is
// first read by the vector ALU at least eight matrix instructions after its last product, or
// behind matrix_result_fence(); registers the vector ALU wrote reach a product behind
// valu_result_fence().
__device__ DBSA_INLINE void mfma_scores_first(floatx16& d, const bf16x8& k, const intx4& q, const floatx16& c) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(d) : "v"(__builtin_bit_cast(intx4, k)), "a"(q), "v"(c));
}
__device__ DBSA_INLINE void mfma_scores_acc(floatx16& d, const bf16x8& k, const intx4& q) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(__builtin_bit_cast(intx4, k)), "a"(q));
}
// mt = max(mt, a, b) on finite-or-infinite inputs (fmaxf would first canonicalise each value that
// comes out of an opaque statement)
__device__ DBSA_INLINE void max3_into(float& mt, float a, float b) {
  asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(mt) : "v"(a), "v"(b));
}
// every pass of a matrix instruction issued before this point has written its result
__device__ DBSA_INLINE void matrix_result_fence() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }
// what the vector ALU wrote before this point may be read by a matrix instruction
__device__ DBSA_INLINE void valu_result_fence() { asm volatile("s_nop 7" ::: "memory"); }

// c ? a : b on VALUES (a conditional on two captured variables is a conditional on their addresses,
// which keeps every variable a lambda captured in memory)
template <typename T>
__device__ DBSA_INLINE T pick(bool c, T a, T b) {
  return c ? a : b;
}

// compile-time description of one step of the pipeline
template <bool QK_, bool SM_, bool PV_, int KBQ_, int KBP_, bool PRE_IN_, bool PRE_OUT_, int DMA_, bool MASK_>
struct StepCfg {
  static constexpr bool QK = QK_, SM = SM_, PV = PV_, PRE_IN = PRE_IN_, PRE_OUT = PRE_OUT_, MASK = MASK_;
  static constexpr int KBQ = KBQ_, KBP = KBP_;  // key half of the score block / of the product block
  // loads spread over the step: 0 none, 1 a K tile, 2 a V tile, 3 / 4 the rows of Q of the next Q tile's
  // first / second row block
  static constexpr int DMA = DMA_;
};

// NW wavefronts per workgroup, each owning row blocks 2*wave and 2*wave+1 of the workgroup's
// 2*NW blocks of 32 rows; row block g covers query head hb * heads_per_block + g / spb (hb = the
// workgroup's head block) and tokens q_start + (g % spb) * 32 .. + 31, spb = block_m / 32.  SL:
// tiles between the issue of a tile's loads and the barrier that publishes them.  SELF: lists may
// name tiles of the call's own K/V (query prefill).
//
// PERSIST = false: one workgroup per (head block, Q tile, run of the tile's list), as in
// attn_prefill.hip.  PERSIST = true: the grid is what the chip holds at once; workgroup w serves
// head block w % n_head_blocks and walks the Q tiles of class w / n_head_blocks of a schedule
// the host balanced (AttnParams::sched_*).  Its K/V tiles form ONE stream across Q tiles: while
// the last tiles of a Q tile are being multiplied, the first tiles of the next one are already on
// their way into the LDS ring, so that a Q tile costs no load latency beyond its own rows of Q.
//
// GATHER (with PERSIST): the rows of a "Q tile" are not consecutive tokens but the references
// gather_refs[q_start .. q_start + q_len), pairs (row of q, slot): row i of the tile is q row
// refs[i][0], and instead of a normalised output the kernel leaves the row's partial softmax state
// (unnormalised accumulators, running maximum, row sum) in partial[slot][head].  This is how a
// decode step with many queries per group runs as a contraction: a record is a run of a group's
// tiles with up to 64 of the queries that selected the group, the four waves are four query heads
// of one KV head, and the merge pass of the decode step combines the slots.
//
// ROPE: Q is un-rotated; the keys carry the rotation of the id they were encoded
// with.  A row is rotated at the id list_shift[e] + (its index inside the Q tile) before it meets
// the keys of list entry e (Sec. 2.2: the retrieved caches get new in-order positions; rotating the
// row instead of the keys lets all queries read the same key bytes).  Entries of one segment share
// the shift, so the fragments are rebuilt only where it changes, from the rows in memory.
// With GATHER (decode step) a record lies inside one segment, so its rows are rotated once, at the record's
// start, each at its own id gather_shift[reference] + self_len[query] - 1.
template <int NW, int SL, bool SELF, bool PERSIST, bool GATHER = false, bool ROPE = false>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_prefill64_kernel(AttnParams p) {
  static_assert(!GATHER || (PERSIST && !SELF), "gathered rows come with a schedule and pool tiles only");
  static_assert(!ROPE || (SELF != GATHER), "rows are re-positioned at the query prefill and at the decode step");
  // the query prefill rotates a Q tile per list entry (the ids ride with the entries); gathered rows are
  // rotated once per record, each at its own id
  constexpr bool kEntryIds = ROPE && !GATHER;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  constexpr int kBlocksPerWave = 16 / NW;  // 1-KiB load blocks of one operand per wave
  constexpr int KS = 2 + SL, VS = 1 + SL;  // LDS stages of K and of V
  static_assert(NW == 2 || NW == 4, "wave count");
  static_assert(SL == 1 || SL == 2 || SL == 3, "load slack");
  const unsigned lds0 = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_byte*)smem));

  const int tid = threadIdx.x, lane = tid % 64, l32 = lane % 32, half = lane / 32;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int r = p.n_q_heads / p.n_kv_heads;
  const int spb = p.block_m / 32;

  // ---- the Q tiles of this workgroup: records (q_start, q_len, first list entry, entries) ----
  const int hb = PERSIST ? static_cast<int>(blockIdx.x) % p.n_head_blocks : static_cast<int>(blockIdx.x);
  int rec_k = 0, rec_end = 1;            // PERSIST: index of the current record in sched_rec, end of the class
  int q_start, q_len, e0, n_tiles;
  if constexpr (PERSIST) {
    const int cls = static_cast<int>(blockIdx.x) / p.n_head_blocks;
    rec_k = __builtin_amdgcn_readfirstlane(p.sched_ptr[cls]);
    rec_end = __builtin_amdgcn_readfirstlane(p.sched_ptr[cls + 1]);
    if (rec_k >= rec_end) return;
    q_start = __builtin_amdgcn_readfirstlane(p.sched_rec[4 * rec_k + 0]);
    q_len = __builtin_amdgcn_readfirstlane(p.sched_rec[4 * rec_k + 1]);
    e0 = __builtin_amdgcn_readfirstlane(p.sched_rec[4 * rec_k + 2]);
    n_tiles = __builtin_amdgcn_readfirstlane(p.sched_rec[4 * rec_k + 3]);
  } else {
    const int tile = __builtin_amdgcn_readfirstlane(p.order[blockIdx.y]);
    q_start = __builtin_amdgcn_readfirstlane(p.qtile_tab[tile * 4 + 0]);
    q_len = __builtin_amdgcn_readfirstlane(p.qtile_tab[tile * 4 + 1]);
    e0 = __builtin_amdgcn_readfirstlane(static_cast<int>(p.list_ptr[tile]));
    n_tiles = __builtin_amdgcn_readfirstlane(static_cast<int>(p.list_ptr[tile + 1])) - e0;
    if (gridDim.z > 1) {
      const int lo = static_cast<int>(static_cast<int64_t>(n_tiles) * blockIdx.z / gridDim.z);
      const int hi = static_cast<int>(static_cast<int64_t>(n_tiles) * (blockIdx.z + 1) / gridDim.z);
      e0 += lo;
      n_tiles = hi - lo;
    }
    if (n_tiles == 0) return;  // the host only cuts lists into non-empty runs
  }
  const const_words sched = (const_words)(reinterpret_cast<uintptr_t>(p.sched_rec));
  const const_words all_ent = (const_words)(reinterpret_cast<uintptr_t>(p.list_ent));
  const const_words all_shift = (const_words)(reinterpret_cast<uintptr_t>(p.list_shift));
  const int hk = (hb * p.heads_per_block) / r;

  const uint64_t kpool = uniform64(reinterpret_cast<uint64_t>(static_cast<const __bf16*>(p.k_pool.ptr) + hk * p.k_pool.stride_head));
  const uint64_t vpool = uniform64(reinterpret_cast<uint64_t>(static_cast<const __bf16*>(p.v_pool.ptr) + hk * p.v_pool.stride_head));
  const uint64_t kself = uniform64(reinterpret_cast<uint64_t>(static_cast<const __bf16*>(p.k_self.ptr) + hk * p.k_self.stride_head));
  const uint64_t vself = uniform64(reinterpret_cast<uint64_t>(static_cast<const __bf16*>(p.v_self.ptr) + hk * p.v_self.stride_head));
  const int kp_stride = static_cast<int>(p.k_pool.stride_tok), vp_stride = static_cast<int>(p.v_pool.stride_tok);
  const int ks_stride = static_cast<int>(p.k_self.stride_tok), vs_stride = static_cast<int>(p.v_self.stride_tok);

  auto decode_ref = [&](int w0, int w1) DBSA_INLINE {
    return TileRef{w0, w1 & 0xFFFF, ((w1 >> 16) & 1) != 0, SELF && ((w1 >> 17) & 1) != 0};
  };

  // ---- global -> LDS loads: this wave fills blocks wave*kBlocksPerWave .. of each operand ----
  // lane -> (row, slot) inside block b: row = 4*b + lane/16, slot = lane%16; the piece fetched
  // into that slot is column (slot ^ swizzle(row)): K by row % 16, V by 4 * (row % 4).
  // The loads a step spreads over its matrix instructions come in groups of four 1-KiB blocks: the first of a
  // group sets the LDS base (m0), the others reach their block with the instruction's offset field, which moves
  // the global address along with the LDS address.  The per-lane offsets therefore carry lane_bias(j) =
  // kDmaBias - 1024 * (j % 4) (never negative, whatever row a lane fetches), and bases are taken kDmaBias lower.
  constexpr unsigned kDmaBias = 3072;
  auto lane_bias = [](int j) { return kDmaBias - 1024u * static_cast<unsigned>(j % 4); };
  unsigned k_lane_off[kBlocksPerWave], v_lane_off[kBlocksPerWave];
#pragma unroll
  for (int j = 0; j < kBlocksPerWave; ++j) {
    const int row_in = 4 * (wave * kBlocksPerWave + j) + lane / 16;
    k_lane_off[j] = static_cast<unsigned>(row_in * kp_stride + (((lane % 16) ^ (row_in % 16)) * 8)) * 2u + lane_bias(j);
    v_lane_off[j] = static_cast<unsigned>(row_in * vp_stride + (((lane % 16) ^ (4 * (row_in % 4))) * 8)) * 2u + lane_bias(j);
  }
  auto issue_k = [&](const TileRef& t, int stage) DBSA_INLINE {
    const uint64_t base = pick(t.self, kself, kpool) + static_cast<uint64_t>(static_cast<unsigned>(t.start)) *
                                                         static_cast<unsigned>(2 * pick(t.self, ks_stride, kp_stride));
    const unsigned dst = lds0 + stage * kTileBytes + wave * kBlocksPerWave * 1024;
    if (__builtin_expect(!t.self && t.len == kBN, 1)) {
#pragma unroll
      for (int j = 0; j < kBlocksPerWave; ++j) dma16(base, k_lane_off[j] - lane_bias(j), dst + j * 1024);
    } else {
      const int stride = pick(t.self, ks_stride, kp_stride);
#pragma unroll
      for (int j = 0; j < kBlocksPerWave; ++j) {
        const int row_in = 4 * (wave * kBlocksPerWave + j) + lane / 16;
        const int row = min(row_in, t.len - 1);  // rows past the tail repeat the last key
        dma16(base, static_cast<unsigned>(row * stride + (((lane % 16) ^ (row_in % 16)) * 8)) * 2u, dst + j * 1024);
      }
    }
  };
  auto issue_v = [&](const TileRef& t, int stage) DBSA_INLINE {
    const uint64_t base = pick(t.self, vself, vpool) + static_cast<uint64_t>(static_cast<unsigned>(t.start)) *
                                                         static_cast<unsigned>(2 * pick(t.self, vs_stride, vp_stride));
    const unsigned dst = lds0 + (KS + stage) * kTileBytes + wave * kBlocksPerWave * 1024;
    if (__builtin_expect(!t.self && t.len == kBN, 1)) {
#pragma unroll
      for (int j = 0; j < kBlocksPerWave; ++j) dma16(base, v_lane_off[j] - lane_bias(j), dst + j * 1024);
    } else {
      const int stride = pick(t.self, vs_stride, vp_stride);
#pragma unroll
      for (int j = 0; j < kBlocksPerWave; ++j) {
        const int row_in = 4 * (wave * kBlocksPerWave + j) + lane / 16;
        const int row = min(row_in, t.len - 1);
        dma16(base, static_cast<unsigned>(row * stride + (((lane % 16) ^ (4 * (row_in % 4))) * 8)) * 2u,
              dst + j * 1024);
      }
    }
  };

  // ---- per-lane LDS read addresses (absolute LDS byte addresses, stage included) ----
  // K fragment (kb, c): row kb*32 + l32, slot (2c + half) ^ (l32 % 16) = k_base ^ (32*c)
  const int k_base = l32 * kRowBytes + ((half ^ (l32 % 16)) * 16);
  // V transpose-read fragment (ob, keys k0..): row k0 + 4*half + j, j = (lane%16)/4; channel
  // slot 4*ob + 2*(l32/16) + (lane%4)/2, swizzled by 4*j; 8-byte half (lane%2) = v_base ^ (64*ob)
  const int v_base = (4 * half + (lane % 16) / 4) * kRowBytes +
                     (((2 * (l32 / 16) + (lane % 4) / 2) ^ (4 * ((lane % 16) / 4))) * 16) + (lane % 2) * 8;
  int kaddr[8], vaddr[4];  // of the K stage / V stage the fragment reads currently walk
#pragma unroll
  for (int c = 0; c < 8; ++c) kaddr[c] = static_cast<int>(lds0) + (k_base ^ (32 * c));
#pragma unroll
  for (int ob = 0; ob < 4; ++ob) vaddr[ob] = static_cast<int>(lds0) + KS * kTileBytes + (v_base ^ (64 * ob));
  int k_rd = 0, v_rd = 0;  // stage the K / V fragment addresses point into
  // K fragment t (t = kb*8 + c); V fragment t (t = kb*8 + ch*4 + ob)
  auto ld_k = [&](auto T) DBSA_INLINE {
    constexpr int t = decltype(T)::value;
    return *(reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(static_cast<uintptr_t>(kaddr[t % 8])) +
             (t / 8) * 32 * kRowBytes / 16);
  };
  auto ld_v = [&](auto T) DBSA_INLINE {
    constexpr int t = decltype(T)::value;
    const lds_byte* vp = reinterpret_cast<const lds_byte*>(static_cast<uintptr_t>(vaddr[t % 4])) +
                         ((t / 8) * 32 + ((t / 4) % 2) * 16) * kRowBytes;
    const bf16x4 lo = lds_read_tr(vp);
    const bf16x4 hi = lds_read_tr(vp + 8 * kRowBytes);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  };
  auto advance_k = [&]() DBSA_INLINE {
    const int k_next = (k_rd + 1 == KS) ? 0 : k_rd + 1;
    const int dk = (k_next - k_rd) * kTileBytes;
#pragma unroll
    for (int c = 0; c < 8; ++c) kaddr[c] += dk;
    k_rd = k_next;
  };
  auto advance_v = [&]() DBSA_INLINE {
    const int v_next = (v_rd + 1 == VS) ? 0 : v_rd + 1;
    const int dv = (v_next - v_rd) * kTileBytes;
#pragma unroll
    for (int ob = 0; ob < 4; ++ob) vaddr[ob] += dv;
    v_rd = v_next;
  };

  // ---- the stream of list entries, across the Q tiles of this workgroup ----
  // f_ent points at the next entry to fetch, f_left counts the entries left in its list; behind a
  // list follows the list of the workgroup's next record.  Behind the last list the stream repeats
  // its last entry: every period loads one K and one V tile, the last ones into stages nobody
  // reads any more, so that the waits can count on a fixed number of loads in flight.
  const_words f_ent = all_ent + 2 * static_cast<int64_t>(e0);
  const_words f_sh = all_shift + (kEntryIds ? static_cast<int64_t>(e0) : 0);  // the entries' rotation ids, in step with f_ent
  int f_left = n_tiles, f_k = rec_k;
  int nx_e0 = 0, nx_n = 0;  // PERSIST: list of record f_k + 1 (requested when the stream entered record f_k)
  if constexpr (PERSIST) {
    if (f_k + 1 < rec_end) {
      nx_e0 = sched[4 * (f_k + 1) + 2];
      nx_n = sched[4 * (f_k + 1) + 3];
    }
  }
  int in_w0 = 0, in_w1 = 0, in_w2 = 0;  // the entry requested last (ROPE: and its rotation id)
  auto request_entry = [&]() DBSA_INLINE {
    if (__builtin_expect(f_left == 0, 0)) {
      if (PERSIST && f_k + 1 < rec_end) {
        f_k += 1;
        f_ent = all_ent + 2 * static_cast<int64_t>(nx_e0);
        if constexpr (kEntryIds) f_sh = all_shift + static_cast<int64_t>(nx_e0);
        f_left = nx_n;
        if (f_k + 1 < rec_end) {
          nx_e0 = sched[4 * (f_k + 1) + 2];
          nx_n = sched[4 * (f_k + 1) + 3];
        }
      } else {
        f_ent -= 2;
        if constexpr (kEntryIds) f_sh -= 1;
        f_left = 1;
      }
    }
    in_w0 = f_ent[0];
    in_w1 = f_ent[1];
    f_ent += 2;
    if constexpr (kEntryIds) {
      in_w2 = f_sh[0];
      f_sh += 1;
    }
    f_left -= 1;
  };

  // (rw0, rw1)[i] = words of the entry i tiles ahead of the one whose scores the current period computes
  int rw0[2 + SL], rw1[2 + SL], rw2[2 + SL];
#pragma unroll
  for (int i = 0; i < 2 + SL; ++i) {
    request_entry();
    rw0[i] = in_w0;
    rw1[i] = in_w1;
    rw2[i] = in_w2;
  }
  // K(0 .. SL) and V(0 .. SL-2) of the stream go out now, in the order later periods keep
  // (K(i), V(i-2)); the period of tile j issues K(j+1+SL) and V(j-1+SL)
  issue_k(decode_ref(rw0[0], rw1[0]), 0);
  issue_k(decode_ref(rw0[1], rw1[1]), 1);
#pragma unroll
  for (int i = 2; i <= SL; ++i) {
    issue_k(decode_ref(rw0[i], rw1[i]), i);
    issue_v(decode_ref(rw0[i - 2], rw1[i - 2]), i - 2);
  }
  int k_wr = (1 + SL) % KS, v_wr = (SL - 1) % VS;  // stages the next period's loads fill

  // ---- per Q tile: rows, Q^T fragments, softmax state ----
  const float c2 = p.scale_log2e;
  int head[2], row_local[2], row_tok[2], q_pos[2];
  int row_slot[2] = {0, 0};  // GATHER: where the row's partial state goes
  int row_rot[2] = {0, 0};   // GATHER with ROPE: the row's rotation id
  bool row_valid[2];
  auto place_rows = [&]() DBSA_INLINE {
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const int g = 2 * wave + rb;
      head[rb] = hb * p.heads_per_block + g / spb;
      row_local[rb] = (g % spb) * 32 + l32;
      row_valid[rb] = row_local[rb] < q_len;
      row_tok[rb] = q_start + min(row_local[rb], q_len - 1);
      q_pos[rb] = q_start + row_local[rb];
      if constexpr (GATHER) {
        // (rows past the last reference repeat it: they compute on its row and store nothing)
        typedef int intx2 __attribute__((ext_vector_type(2)));
        const intx2 ref = *reinterpret_cast<const intx2*>(p.gather_refs + 2 * static_cast<int64_t>(row_tok[rb]));
        if constexpr (ROPE)  // the decode row of query ref[0] sits at index self_len - 1 of its own cache
          row_rot[rb] = p.gather_shift[row_tok[rb]] + p.self_len[ref[0]] - 1;
        row_tok[rb] = ref[0];
        row_slot[rb] = ref[1];
      }
    }
  };
  // A lane's row of Q arrives as eight 16-byte pieces (32 rows per load instruction, two pieces each: the
  // address unit spends tens of cycles on every one).  The first Q tile's are requested in one go; those
  // of a following Q tile ride on the drain steps of the one before, one piece every other matrix instruction.
  bf16x8 q_raw[2][kD / 16];
  const __bf16* q_next[2];
  auto aim_q = [&]() DBSA_INLINE {
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
      q_next[rb] = static_cast<const __bf16*>(p.q.ptr) + static_cast<int64_t>(row_tok[rb]) * p.q.stride_tok +
                   static_cast<int64_t>(head[rb]) * p.q.stride_head + 8 * half;
  };
  auto load_q = [&]() DBSA_INLINE {
    aim_q();
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int c = 0; c < kD / 16; ++c) q_raw[rb][c] = *reinterpret_cast<const bf16x8*>(q_next[rb] + 16 * c);
  };
  intx4 qf[2][kD / 16];  // Q^T fragments pre-multiplied by scale*log2(e), in accumulation registers
  auto scale_q = [&]() DBSA_INLINE {
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int c = 0; c < kD / 16; ++c) {
        union {
          bf16x8 v;
          bf16x2 p2[4];
        } sc;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          sc.p2[e] = __builtin_convertvector(floatx2{static_cast<float>(q_raw[rb][c][2 * e]) * c2,
                                                     static_cast<float>(q_raw[rb][c][2 * e + 1]) * c2}, bf16x2);
        qf[rb][c] = __builtin_bit_cast(intx4, sc.v);
        asm volatile("" : "+a"(qf[rb][c]));
      }
    valu_result_fence();
  };
  // ROPE: the fragments of both row blocks from the rows in memory, rotated at shift + row index and
  // pre-multiplied like scale_q's (rare: once per segment of a list)
  int cur_shift = 0;
  auto rotate_q = [&](int shift) DBSA_INLINE {
    cur_shift = shift;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const __bf16* qp = static_cast<const __bf16*>(p.q.ptr) + static_cast<int64_t>(row_tok[rb]) * p.q.stride_tok +
                         static_cast<int64_t>(head[rb]) * p.q.stride_head + 8 * half;
      const int id = min(max(GATHER ? row_rot[rb] : shift + row_local[rb], 0), p.rope_n_pos - 1);
      const float* rot = p.rope_table + static_cast<int64_t>(id) * kD + 16 * half;
      bf16x8 frag[kD / 16];
      load_query_fragments<true>(qp, rot, c2, frag);
#pragma unroll
      for (int c = 0; c < kD / 16; ++c) {
        qf[rb][c] = __builtin_bit_cast(intx4, frag[c]);
        asm volatile("" : "+a"(qf[rb][c]));
      }
    }
    valu_result_fence();
  };
  place_rows();
  if constexpr (!ROPE) load_q();

  floatx16 o[2][kD / 32];
  floatx16 neg_m[2];                     // minus the running maximum in every element: C operand of a score block's first product
  float m_run[2], l_run[2];              // running max (log2 domain, meaningful once seen); this lane's share of the row sum
  bool seen[2];                          // the row has met a visible key

  // masks of a causal or short tile, applied to the scores of its key half kb
  auto apply_mask = [&](floatx16 (&s)[2], const TileRef& t, int kb) DBSA_INLINE {
    int key0 = 4 * half + 32 * kb;
    asm volatile("" : "+v"(key0));  // keeps loop-invariant key indices out of registers: this path is rare
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      // element i holds key key0 + 8 * (i / 4) + i % 4 of the tile; it is visible iff that index is below the
      // tile's length and (causal tiles) not beyond the row's own position: one bound per lane, relative to key0
      const int last = min(t.causal ? (q_pos[rb] - t.start) : kBN, t.len - 1) - key0;
      // (a row block that sees all 32 keys of this half needs nothing: 27 is the largest element offset)
      if (__builtin_amdgcn_ballot_w64(last < 27) == 0) continue;
#pragma unroll
      for (int i = 0; i < 16; ++i) s[rb][i] = (8 * (i / 4) + (i % 4)) <= last ? s[rb][i] : -INFINITY;
    }
  };

  floatx16 s_e[2], s_o[2];         // scores (minus running max) of even / odd half tiles
  bf16x2 p_e[2][8], p_o[2][8];     // their probabilities, packed as B operands of the second product
  bf16x8 ring[kRing];
  float ls[2];                     // this lane's sum of the probabilities of the latest step, not yet in l_run
  bool all_seen;                   // wave-uniform: every row of the wave has met a visible key
  // loads a step spreads over its matrix instructions: global base, LDS address of the wave's first block
  uint64_t dma_base = 0;
  unsigned dma_dst = 0;

  // exact row maximum of 32 x 32 scores (this lane's 16 values, then the other key half)
  auto row_max = [&](const floatx16& sc) DBSA_INLINE {
    float mt = kNoKey;
#pragma unroll
    for (int i = 0; i < 8; ++i) max3_into(mt, sc[2 * i], sc[2 * i + 1]);
    return half_swap_max(mt);
  };

  // One step.  QK: S_w = scores of half tile h+1 (key half KBQ of the K stage the addresses walk).
  // SM: P_w = probabilities of half tile h from S_r.  PV: O += V P_r for half tile h-1 (key half
  // KBP of the V stage); on entry S_w still holds the scores P_r was made from.  PRE_IN: the ring
  // already holds the step's first kDist fragments.  PRE_OUT: on exit it holds the first kDist K
  // fragments of the next step.  DMA: 1 = spread this wave's share of a K tile (dma_base, dma_dst)
  // over the step, 2 = of a V tile, 3 / 4 = the rows of Q at q_next[0] / q_next[1] into q_raw.  MASK: the
  // scores of this step may need the mask of tile tq.
  auto step = [&](auto CFG, floatx16 (&S_w)[2], floatx16 (&S_r)[2], bf16x2 (&P_w)[2][8], bf16x2 (&P_r)[2][8],
                  const TileRef& tq) DBSA_INLINE {
    using C = decltype(CFG);
    constexpr int nK = C::QK ? 8 : 0, nV = C::PV ? 8 : 0, nF = nK + nV, nSlots = 2 * nF;
    constexpr int nRead = nF + (C::PRE_OUT ? kDist : 0);  // fragments this step reads from LDS, its own first
    static_assert(nF % kRing == 0 && kDist < kRing, "ring slots carry over from step to step");

    // No row maxima are taken on the way: a row's running maximum only has to bound its scores
    // to within what bf16 and fp32 hold, and the sum of a step's probabilities shows when it no
    // longer does.  rare: the probabilities made in the previous step came out too large (one of
    // them may even be infinite): make them again around the true maximum, before they are used.
    if constexpr (C::PV) {
      const bool big = ls[0] + ls[1] > kOverflowSum;  // all terms are positive or zero
      if (__builtin_expect(__builtin_amdgcn_ballot_w64(big) != 0, 0)) {
        matrix_result_fence();
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          const float delta = __builtin_ceilf(fmaxf(row_max(S_w[rb]), 0.f));  // whole log2 units
          const float alpha = __builtin_amdgcn_exp2f(-delta);
          m_run[rb] += delta;
          l_run[rb] *= alpha;
          // the accumulators live in accumulation registers; the opaque statements pin the copies to
          // and from ordinary registers inside this rare block (the compiler otherwise hoists them
          // to the head of the tile loop)
#pragma unroll
          for (int ob = 0; ob < kD / 32; ++ob) {
            asm volatile("" : "+a"(o[rb][ob]));
            o[rb][ob] *= alpha;
            asm volatile("" : "+a"(o[rb][ob]));
          }
          float sum = 0.f;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float x0 = __builtin_amdgcn_exp2f(S_w[rb][2 * e] - delta), x1 = __builtin_amdgcn_exp2f(S_w[rb][2 * e + 1] - delta);
            P_r[rb][e] = __builtin_convertvector(floatx2{x0, x1}, bf16x2);
            sum += x0 + x1;
          }
          ls[rb] = sum;
#pragma unroll
          for (int i = 0; i < 16; ++i) S_r[rb][i] -= delta;
#pragma unroll
          for (int i = 0; i < 16; ++i) neg_m[rb][i] -= delta;
        }
        valu_result_fence();
      }
      l_run[0] += ls[0];
      l_run[1] += ls[1];
      ls[0] = 0.f;
      ls[1] = 0.f;
    }
    // rare (the first step of every list): rows that have met no visible key yet take their running
    // maximum from the scores about to become probabilities; their sums and outputs are still zero
    if constexpr (C::SM) {
      if (__builtin_expect(!all_seen, 0)) {
        matrix_result_fence();
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          const float m_true = row_max(S_r[rb]);
          const bool first = !seen[rb] & (m_true > kNoKey);
          const float delta = first ? __builtin_ceilf(m_true) : 0.f;
          seen[rb] = seen[rb] | first;
          m_run[rb] += delta;
#pragma unroll
          for (int i = 0; i < 16; ++i) S_r[rb][i] -= delta;
#pragma unroll
          for (int i = 0; i < 16; ++i) neg_m[rb][i] -= delta;
        }
        all_seen = __builtin_amdgcn_ballot_w64(!seen[0] | !seen[1]) == 0;
        valu_result_fence();
      }
    }

    // fragment i of this step: K fragments of the score block, then V fragments of the product
    // block, then (PRE_OUT) the first K fragments of the next step's score block
    auto read_frag = [&](auto I) DBSA_INLINE {
      constexpr int i = decltype(I)::value;
      if constexpr (i < nK)
        ring[i % kRing] = ld_k(std::integral_constant<int, C::KBQ * 8 + i>{});
      else if constexpr (i < nF)
        ring[i % kRing] = ld_v(std::integral_constant<int, C::KBP * 8 + (i - nK)>{});
      else
        ring[i % kRing] = ld_k(std::integral_constant<int, (C::QK ? 1 - C::KBQ : 0) * 8 + (i - nF)>{});
    };
    if constexpr (!C::PRE_IN) static_for<(kDist < nRead ? kDist : nRead)>([&](auto I) DBSA_INLINE { read_frag(I); });

    float ee[2][2] = {{0.f, 0.f}, {0.f, 0.f}};  // exponentials of units u and u-1: a unit is packed behind the next one's
    auto pack_unit = [&](auto U) DBSA_INLINE {
      constexpr int u = decltype(U)::value;
      P_w[u / 8][u % 8] = __builtin_convertvector(floatx2{ee[u % 2][0], ee[u % 2][1]}, bf16x2);
      ls[u / 8] += ee[u % 2][0] + ee[u % 2][1];
      asm volatile("" : "+v"(P_w[u / 8][u % 8]), "+v"(ls[u / 8]));
    };
    __builtin_amdgcn_sched_barrier(0);
    static_for<nSlots>([&](auto T) DBSA_INLINE {
      constexpr int t = decltype(T)::value, f = t / 2, rb = t % 2;
      // ---- matrix instruction of this slot ----
      if constexpr (f < nK) {
        if constexpr (f == 0)
          mfma_scores_first(S_w[rb], ring[f % kRing], qf[rb][f], neg_m[rb]);
        else
          mfma_scores_acc(S_w[rb], ring[f % kRing], qf[rb][f]);
      } else {
        constexpr int g = f - nK, ch = g / 4, ob = g % 4;
        union {
          bf16x8 v;
          bf16x2 p2[4];
        } pf;
#pragma unroll
        for (int e = 0; e < 4; ++e) pf.p2[e] = P_r[rb][4 * ch + e];
        o[rb][ob] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[f % kRing], pf.v, o[rb][ob], 0, 0, 0);
      }
      // ---- fragment read kDist fragments ahead ----
      if constexpr (rb == 0) {
        // the K addresses move on to the next stage once the last fragment of key half 1 is requested
        if constexpr (C::QK && C::KBQ == 1 && f + kDist == nK) advance_k();
        if constexpr (f + kDist < nRead) read_frag(std::integral_constant<int, f + kDist>{});
      }
      // ---- this wave's loads of the period, one every few matrix instructions ----
      if constexpr (C::DMA == 1 || C::DMA == 2) {
        constexpr int every = nSlots / kBlocksPerWave;
        if constexpr (t % every == every - 1)
        {
          constexpr int b = t / every;
          const unsigned off = C::DMA == 1 ? k_lane_off[b] : v_lane_off[b];
          if constexpr (b % 4 == 0)
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                         :
                         : "s"(dma_dst + b * 1024), "v"(off), "s"(dma_base)
                         : "memory");
          else  // (nothing between the loads of a group writes m0: LDS reads do not use it on this chip)
            asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" : : "v"(off), "s"(dma_base), "n"((b % 4) * 1024) : "memory");
        }
      }
      if constexpr (C::DMA == 3 || C::DMA == 4) {
        static_assert(C::DMA < 3 || nSlots == 2 * (kD / 16), "one piece of Q every other slot");
        if constexpr (t % 2 == 1) q_raw[C::DMA - 3][t / 2] = *reinterpret_cast<const bf16x8*>(q_next[C::DMA - 3] + 16 * (t / 2));
      }
      // ---- vector work in the shadow of the matrix instruction ----
      if constexpr (C::SM) {
        // 16 units (8 per row block) of two exponentials.  A full step has two slots per unit: one
        // exponential in each, and behind it one half of the previous unit's packing (a result of the
        // transcendental unit cannot be used by the very next instructions), so that every matrix
        // instruction shadows about the same vector work.  A short step has one slot per unit.
        if constexpr (nSlots >= 32) {
          constexpr int u = t / 2, w = t % 2;
          ee[u % 2][w] = __builtin_amdgcn_exp2f(S_r[u / 8][2 * (u % 8) + w]);
          asm volatile("" : "+v"(ee[u % 2][w]));
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (u > 0) {
            constexpr int pu = u - 1;
            if constexpr (w == 0) {
              ls[pu / 8] += ee[pu % 2][0];
              asm volatile("" : "+v"(ls[pu / 8]));
            } else {
              P_w[pu / 8][pu % 8] = __builtin_convertvector(floatx2{ee[pu % 2][0], ee[pu % 2][1]}, bf16x2);
              ls[pu / 8] += ee[pu % 2][1];
              asm volatile("" : "+v"(P_w[pu / 8][pu % 8]), "+v"(ls[pu / 8]));
            }
          }
        } else {
          constexpr int u = t;
          ee[u % 2][0] = __builtin_amdgcn_exp2f(S_r[u / 8][2 * (u % 8)]);
          ee[u % 2][1] = __builtin_amdgcn_exp2f(S_r[u / 8][2 * (u % 8) + 1]);
          asm volatile("" : "+v"(ee[u % 2][0]), "+v"(ee[u % 2][1]));
          // the previous unit is packed behind these exponentials
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (u > 0) pack_unit(std::integral_constant<int, u - 1>{});
        }
      }
      if constexpr (C::QK && C::MASK && nSlots >= 32 && t == 24) {
        // the new scores' last product is eight matrix instructions back
        if (__builtin_expect(tq.causal || tq.len < kBN, 0)) apply_mask(S_w, tq, C::KBQ);
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    if constexpr (C::SM) pack_unit(std::integral_constant<int, 15>{});
    if constexpr (C::QK && nSlots < 32) {
      // a short step: the next step reads these scores right away
      matrix_result_fence();
      if constexpr (C::MASK) {
        if (__builtin_expect(tq.causal || tq.len < kBN, 0)) apply_mask(S_w, tq, C::KBQ);
      }
    }
    if constexpr (C::PV && C::KBP == 1) advance_v();
  };

  // The per-lane offsets of a tile's loads (k_lane_off, v_lane_off) are those of a whole pool tile;
  // a short tile or a tile of the call's own K/V gets its own for the period that loads it.
  bool k_special = false, v_special = false;
  auto lane_offsets = [&](unsigned (&off)[kBlocksPerWave], const TileRef& t, int stride, bool for_v) DBSA_INLINE {
#pragma unroll
    for (int i = 0; i < kBlocksPerWave; ++i) {
      const int row_in = 4 * (wave * kBlocksPerWave + i) + lane / 16;
      const int row = min(row_in, t.len - 1);  // rows past the tail repeat the last key
      const int sw = for_v ? 4 * (row_in % 4) : row_in % 16;
      off[i] = static_cast<unsigned>(row * stride + (((lane % 16) ^ sw) * 8)) * 2u + lane_bias(i);
    }
  };
  // the K tile (entry 1+SL ahead) / the V tile (entry SL-1 ahead) a period loads
  auto aim_k = [&]() DBSA_INLINE {
    const TileRef tk = decode_ref(rw0[1 + SL], rw1[1 + SL]);
    const bool special = tk.self || tk.len != kBN;
    if (__builtin_expect(special || k_special, 0)) lane_offsets(k_lane_off, tk, pick(tk.self, ks_stride, kp_stride), false);
    k_special = special;
    // (made uniform again by hand: under register pressure the compiler forms these with vector
    // instructions, and the load instruction takes them in scalar registers only)
    dma_base = uniform64(pick(tk.self, kself, kpool) + static_cast<uint64_t>(static_cast<unsigned>(tk.start)) *
                                                           static_cast<unsigned>(2 * pick(tk.self, ks_stride, kp_stride)) -
                         kDmaBias);
    dma_dst = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(
        static_cast<int>(lds0 + k_wr * kTileBytes + wave * kBlocksPerWave * 1024)));
  };
  auto aim_v = [&]() DBSA_INLINE {
    const TileRef tv = decode_ref(rw0[SL - 1], rw1[SL - 1]);
    const bool special = tv.self || tv.len != kBN;
    if (__builtin_expect(special || v_special, 0)) lane_offsets(v_lane_off, tv, pick(tv.self, vs_stride, vp_stride), true);
    v_special = special;
    dma_base = uniform64(pick(tv.self, vself, vpool) + static_cast<uint64_t>(static_cast<unsigned>(tv.start)) *
                                                           static_cast<unsigned>(2 * pick(tv.self, vs_stride, vp_stride)) -
                         kDmaBias);
    dma_dst = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(
        static_cast<int>(lds0 + (KS + v_wr) * kTileBytes + wave * kBlocksPerWave * 1024)));
  };
  // the end of a period that computed scores: the queue moves on by one entry
  auto next_period = [&]() DBSA_INLINE {
#pragma unroll
    for (int i = 0; i < 1 + SL; ++i) {
      rw0[i] = rw0[i + 1];
      rw1[i] = rw1[i + 1];
      if constexpr (kEntryIds) rw2[i] = rw2[i + 1];
    }
    rw0[1 + SL] = in_w0;
    rw1[1 + SL] = in_w1;
    if constexpr (kEntryIds) rw2[1 + SL] = in_w2;
    k_wr = (k_wr + 1 == KS) ? 0 : k_wr + 1;
    v_wr = (v_wr + 1 == VS) ? 0 : v_wr + 1;
  };
  // A barrier between two periods publishes the K tile one ahead of the next period's and the V
  // tile the next period multiplies, both issued SL periods earlier; the loads of the SL-1 periods
  // since may stay in flight.  (A bare barrier: the LDS reads still in flight here are the next
  // step's first fragments, of a stage nobody refills yet; the wait's memory clobber keeps the
  // compiler from moving LDS reads across.)
  auto period_barrier = [&]() DBSA_INLINE {
    wait_vmcnt<2 * (SL - 1) * kBlocksPerWave>();
    __builtin_amdgcn_s_barrier();
  };

  for (;;) {
    // ---- a Q tile: its rows of Q are in q_raw (requested before the previous tile's epilogue) ----
    if constexpr (ROPE)
      rotate_q(kEntryIds ? rw2[0] : 0);
    else
      scale_q();
    int nq_start = 0, nq_len = 0, nq_e0 = 0, nq_n = 0;  // PERSIST: the record after this one
    if constexpr (PERSIST) {
      if (rec_k + 1 < rec_end) {
        nq_start = sched[4 * (rec_k + 1) + 0];
        nq_len = sched[4 * (rec_k + 1) + 1];
        nq_e0 = sched[4 * (rec_k + 1) + 2];
        nq_n = sched[4 * (rec_k + 1) + 3];
      }
    }
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
      for (int ob = 0; ob < kD / 32; ++ob)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[rb][ob][i] = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) neg_m[rb][i] = 0.f;
      m_run[rb] = 0.f;
      l_run[rb] = 0.f;
      ls[rb] = 0.f;
      seen[rb] = false;
    }
    all_seen = false;

    // ---- period 0: scores of both halves of tile 0, probabilities of the first ----
    // (its loads ride on its steps like those of the later periods: the per-lane offsets may still
    // be those of a special tile the previous Q tile loaded last, which aim_k / aim_v put right)
    period_barrier();
    request_entry();
    {
      const TileRef t0 = decode_ref(rw0[0], rw1[0]);
      aim_k();
      step(StepCfg<true, false, false, 0, 0, false, false, 1, true>{}, s_e, s_o, p_o, p_e, t0);
      aim_v();
      step(StepCfg<true, true, false, 1, 0, false, true, 2, true>{}, s_o, s_e, p_e, p_o, t0);
    }
    next_period();

    // ---- periods 1 .. n_tiles-1: the steady state ----
    for (int j = 1; j < n_tiles; ++j) {
      request_entry();  // before the barrier, whose wait covers the entry's latency
      period_barrier();
      const TileRef tq = decode_ref(rw0[0], rw1[0]);
      if constexpr (kEntryIds) {
        // this period computes the scores of an entry of another segment: rebuild Q for it (every matrix
        // instruction that read the old fragments was issued a period ago)
        if (__builtin_expect(rw2[0] != cur_shift, 0)) rotate_q(rw2[0]);
      }
      aim_k();
      step(StepCfg<true, true, true, 0, 0, true, true, 1, true>{}, s_e, s_o, p_o, p_e, tq);
      aim_v();
      step(StepCfg<true, true, true, 1, 1, true, true, 2, true>{}, s_o, s_e, p_e, p_o, tq);
      next_period();
    }

    // ---- drain: the last tile's second probabilities and both of its products (no loads) ----
    period_barrier();
    // the rows this Q tile writes; then the next Q tile's rows of Q are requested along the drain steps,
    // and arrive during the epilogue
    const int o_start = q_start, o_len = q_len;
    int o_head[2], o_tok[2], o_slot[2];
    bool o_valid[2];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      o_head[rb] = head[rb];
      o_tok[rb] = row_tok[rb];
      o_slot[rb] = row_slot[rb];
      o_valid[rb] = row_valid[rb];
    }
    const bool more = PERSIST && rec_k + 1 < rec_end;
    if (more) {
      rec_k += 1;
      q_start = nq_start;
      q_len = nq_len;
      e0 = nq_e0;
      n_tiles = nq_n;
      place_rows();
    }
    {
      // (no Q tile follows: the pieces of the current rows come once more, into registers nobody reads)
      constexpr int kQ0 = ROPE ? 0 : 3, kQ1 = ROPE ? 0 : 4;
      if constexpr (!ROPE) aim_q();
      const TileRef none{0, kBN, false, false};
      step(StepCfg<false, true, true, 0, 0, false, false, kQ0, false>{}, s_e, s_o, p_o, p_e, none);
      step(StepCfg<false, false, true, 0, 1, false, false, kQ1, false>{}, s_o, s_e, p_e, p_o, none);
    }
    // the sums of the last step (a sum that is too large is caught by the product step after it, and
    // the last one is followed by none)
    l_run[0] += ls[0];
    l_run[1] += ls[1];

    // ---- epilogue ----
    if constexpr (GATHER) {
      // Partial states, 528-byte rows of fp32: like the normalised outputs below they go through LDS
      // so that a store instruction writes whole 256-byte pieces of four rows instead of 16 bytes of
      // each of 32 rows; a row block passes in two halves of 64 channels, 8 KiB of staging per wave.
      __builtin_amdgcn_s_barrier();
      const int k_last = (k_rd == 0 ? KS : k_rd) - 1, v_last = (v_rd == 0 ? VS : v_rd) - 1;
      const bool in_k = (NW == 4 ? wave / 2 : wave) == 0;
      const unsigned stag = lds0 + (in_k ? k_last : KS + v_last) * kTileBytes + (NW == 4 ? (wave % 2) * 8192 : 0);
      typedef __attribute__((address_space(3))) floatx4* lds_f128;
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
        const float l_tot = half_swap_sum(l_run[rb]);
        float* head_base = p.partial + static_cast<int64_t>(o_head[rb]) * (kD + kPartialPad) + (lane % 16) * 4;
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
#pragma unroll
          for (int ob2 = 0; ob2 < 2; ++ob2)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              const int ob = 2 * h2 + ob2;
              *(lds_f128)(static_cast<uintptr_t>(stag + l32 * kRowBytes + (((8 * ob2 + 2 * g + half) ^ (l32 % 16)) * 16))) =
                  floatx4{o[rb][ob][4 * g], o[rb][ob][4 * g + 1], o[rb][ob][4 * g + 2], o[rb][ob][4 * g + 3]};
            }
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const int row = 4 * i + lane / 16;
            const floatx4 piece = *(lds_f128)(static_cast<uintptr_t>(stag + row * kRowBytes + (((lane % 16) ^ (row % 16)) * 16)));
            // the slot of that row is held by the lane that owns the row
            const int slot = __builtin_amdgcn_ds_bpermute(4 * row, o_slot[rb]);
            if (32 * rb + row < o_len)
              *reinterpret_cast<floatx4*>(head_base + static_cast<int64_t>(slot) * p.n_q_heads * (kD + kPartialPad) + 64 * h2) = piece;
          }
        }
        if (half == 0 && o_valid[rb]) {
          float* part = p.partial + (static_cast<int64_t>(o_slot[rb]) * p.n_q_heads + o_head[rb]) * (kD + kPartialPad);
          part[kD] = seen[rb] ? m_run[rb] : -1.0e30f;
          part[kD + 1] = l_tot;
        }
      }
    } else if (!PERSIST && gridDim.z > 1) {
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
        const float l_tot = half_swap_sum(l_run[rb]);
        if (!o_valid[rb]) continue;
        float* part = p.partial + ((static_cast<int64_t>(o_tok[rb]) * p.n_q_heads + o_head[rb]) * gridDim.z + blockIdx.z) *
                                      (kD + kPartialPad);
#pragma unroll
        for (int ob = 0; ob < kD / 32; ++ob)
#pragma unroll
          for (int g = 0; g < 4; ++g)
            *reinterpret_cast<floatx4*>(part + 32 * ob + 8 * g + 4 * half) =
                floatx4{o[rb][ob][4 * g], o[rb][ob][4 * g + 1], o[rb][ob][4 * g + 2], o[rb][ob][4 * g + 3]};
        if (half == 0) {
          // a run none of whose keys the row may see contributes nothing: the merge weighs it with 2^(m - m*)
          part[kD] = seen[rb] ? m_run[rb] : -1.0e30f;
          part[kD + 1] = l_tot;
        }
      }
    } else {
      // A lane holds one row's channels four at a time, so stores from the registers would write 16
      // bytes to each of 32 rows per instruction.  The rows go through LDS instead and leave as whole
      // 256-byte rows, four per instruction: each wave turns its two row blocks around in 8 KiB of
      // the stages of the last K and V tiles, which nobody reads after the barrier below and which
      // are refilled only behind the next period's barrier.  Row r keeps its 16-byte pieces XOR-ed
      // with r % 16, so that both the writes (one row per lane) and the reads (16 lanes per row)
      // spread over all banks.
      __builtin_amdgcn_s_barrier();
      const int k_last = (k_rd == 0 ? KS : k_rd) - 1, v_last = (v_rd == 0 ? VS : v_rd) - 1;
      const bool in_k = (NW == 4 ? wave / 2 : wave) == 0;
      const unsigned stag = lds0 + (in_k ? k_last : KS + v_last) * kTileBytes + (NW == 4 ? (wave % 2) * 8192 : 0);
      typedef __attribute__((address_space(3))) bf16x4* lds_b64;
      typedef __attribute__((address_space(3))) intx4* lds_b128;
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
        const float l_tot = half_swap_sum(l_run[rb]);
        const float inv = 1.f / l_tot;
#pragma unroll
        for (int ob = 0; ob < kD / 32; ++ob)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            union {
              bf16x4 v;
              bf16x2 p2[2];
            } w;
            w.p2[0] = __builtin_convertvector(floatx2{o[rb][ob][4 * g] * inv, o[rb][ob][4 * g + 1] * inv}, bf16x2);
            w.p2[1] = __builtin_convertvector(floatx2{o[rb][ob][4 * g + 2] * inv, o[rb][ob][4 * g + 3] * inv}, bf16x2);
            *(lds_b64)(static_cast<uintptr_t>(stag + l32 * kRowBytes + (((4 * ob + g) ^ (l32 % 16)) * 16) + half * 8)) = w.v;
          }
        const int row_base = ((2 * wave + rb) % spb) * 32;
        __bf16* op = static_cast<__bf16*>(const_cast<void*>(p.o.ptr)) + static_cast<int64_t>(o_head[rb]) * p.o.stride_head +
                     (lane % 16) * 8;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int row = 4 * i + lane / 16;
          const intx4 piece = *(lds_b128)(static_cast<uintptr_t>(stag + row * kRowBytes + (((lane % 16) ^ (row % 16)) * 16)));
          if (row_base + row < o_len)
            *reinterpret_cast<intx4*>(op + static_cast<int64_t>(o_start + row_base + row) * p.o.stride_tok) = piece;
        }
        if (p.lse && half == 0 && o_valid[rb])
          p.lse[static_cast<int64_t>(o_head[rb]) * p.lse_stride + o_tok[rb]] = (m_run[rb] + __log2f(l_tot)) * 0.69314718055994531f;
      }
    }
    if (!more) break;
  }
}

template <int NW, int SL, bool SELF, bool PERSIST, bool GATHER = false, bool ROPE = false>
hipError_t launch_cfg64(const AttnParams& p, hipStream_t stream) {
  constexpr int lds_bytes = (3 + 2 * SL) * kTileBytes;
  static std::atomic<bool> attr_set{false};  // setting it twice from two threads is harmless
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_prefill64_kernel<NW, SL, SELF, PERSIST, GATHER, ROPE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int n_split = p.q_split > 1 ? p.q_split : 1;
  const dim3 grid = PERSIST ? dim3(p.sched_classes * p.n_head_blocks)
                            : dim3(p.n_q_heads / p.heads_per_block, p.n_qtiles, n_split);
  attn_prefill64_kernel<NW, SL, SELF, PERSIST, GATHER, ROPE><<<grid, dim3(NW * 64), lds_bytes, stream>>>(p);
  return hipGetLastError();
}

template <int NW, int SL>
hipError_t launch_stage64(const AttnParams& p, hipStream_t stream) {
  if (p.rope_table) {
    if (!p.query_stage || !p.list_shift) return hipErrorInvalidValue;
    return p.sched_rec ? launch_cfg64<NW, SL, true, true, false, true>(p, stream)
                       : launch_cfg64<NW, SL, true, false, false, true>(p, stream);
  }
  if (p.sched_rec)
    return p.query_stage ? launch_cfg64<NW, SL, true, true>(p, stream) : launch_cfg64<NW, SL, false, true>(p, stream);
  return p.query_stage ? launch_cfg64<NW, SL, true, false>(p, stream) : launch_cfg64<NW, SL, false, false>(p, stream);
}

}  // namespace

// Eight row blocks per workgroup: four waves alone on a compute unit (112 KiB of LDS, two tiles
// of load slack); four row blocks: two waves, two workgroups per compute unit (80 KiB each).
// With a schedule in p (sched_rec) the launch is persistent and p.q_split must be 1.  The caller
// runs the merge pass of a split launch.
hipError_t launch_prefill64(const AttnParams& p, hipStream_t stream) {
  if (p.n_qtiles == 0) return hipSuccess;
  const int row_blocks = p.heads_per_block * (p.block_m / 32);
  switch (row_blocks) {
    case 4: return launch_stage64<2, 1>(p, stream);
    case 8: return launch_stage64<4, 2>(p, stream);
    default: return hipErrorInvalidValue;
  }
}

// The pool items of a decode step as a contraction: p carries the schedule of the layout's matrix
// records (sched_*), the segments' tile entries as list_ent, the flat references as gather_refs and
// the decode step's q, pools and partial buffer; query heads in fours per KV head, 64-row tiles.
hipError_t launch_decode_matrix_items(const AttnParams& p, hipStream_t stream) {
  if (!p.sched_rec || !p.sched_ptr || !p.gather_refs || !p.partial || p.sched_classes < 1) return hipErrorInvalidValue;
  if (p.heads_per_block != 4 || p.block_m != 64 || p.n_q_heads % (4 * p.n_kv_heads) != 0 || p.n_head_blocks != p.n_q_heads / 4)
    return hipErrorInvalidValue;
  if (p.rope_table) {
    if (!p.gather_shift || !p.self_len) return hipErrorInvalidValue;
    return launch_cfg64<4, 2, false, true, true, true>(p, stream);
  }
  return launch_cfg64<4, 2, false, true, true>(p, stream);
}
