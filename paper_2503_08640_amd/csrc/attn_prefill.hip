// Software-pipelined bf16 MFMA attention for prefill-shaped calls (pre-encode, Sec. 2.1;
// query prefill, Sec. 2.2) at head_dim 128 on gfx950.  Same mathematics and register
// plan as attn_mfma.hip (transposed scores S^T = K Q^T, per-lane softmax statistics,
// O^T = V^T P^T).  The kernel is organised so that a wavefront never waits on a latency
// inside a KV tile: between two workgroup barriers it runs 32 matrix instructions, each
// followed by the few vector instructions that fit in its shadow.
//
//   * K and V tiles go from global memory straight into LDS with
//     global_load_lds_dwordx4 (no staging registers, no ds_write).  A wave-level load
//     fills 1 KiB of LDS in lane order, so the layout is unpadded and bank conflicts are
//     avoided by choosing WHICH 16-byte piece each lane fetches: row-major 256-byte rows
//     whose 16-byte slots are XOR-swizzled, K by (row % 16) for the 128-bit fragment
//     reads (16 consecutive rows, same slot -> 16 distinct bank groups) and V by
//     4*(row % 4) for the 64-bit transpose reads (4 rows x 4 slots per half-wave).
//   * tiles are fetched SL steps before the barrier that publishes them (2 + SL stages of
//     K, 1 + SL of V) and K becomes visible one barrier before its scores are computed:
//     a step is  [barrier]  S(j+1) = K(j+1) Q^T  |  O += V(j) P(j)  and the operand
//     fragments of a step's first matrix instructions are already in registers when the
//     barrier opens (they were read from LDS at the end of the previous step).
//   * operand fragments travel through one ring of registers, read from LDS kRing - 1
//     matrix instructions ahead of their use, across the K -> V -> next-K boundaries.
//   * Q is pre-multiplied by scale*log2(e) when its fragments are loaded, and the score
//     accumulators start at minus the running row maximum (the C operand of a score block's
//     first matrix instruction is a register block holding it), so that a probability is one
//     v_exp_f32 of the MFMA result; the row sum is accumulated in fp32 with plain adds
//     (v_dot2c_f32_bf16 with a vector of ones would be fewer instructions, but measured it
//     stalls ~15 cycles behind every MFMA in flight: dot instructions share the matrix pipe).
//   * the exponentials of tile j are issued in the shadow of the score MFMAs of tile j+1,
//     their packing one MFMA later; row maxima of tile j+1 and the initialisation of the
//     next score accumulators ride on the second product.
//   * the running maximum may lag the true maximum by kRescaleSlack (weights then reach
//     2^slack at most, harmless in fp32/bf16): accumulators are rescaled only when some
//     row of the wave outgrows it, which is rare once a few tiles have been seen.
#include <atomic>
#include <cstdint>
#include <type_traits>
#include <utility>

#include "kernels.hpp"
#include "mfma_common.hpp"

namespace {

using namespace dbsa_mfma;

constexpr int kD = 128;
constexpr int kBN = 64;                       // keys per KV tile
constexpr int kRowBytes = kD * 2;             // 256
constexpr int kTileBytes = kBN * kRowBytes;   // 16 KiB per K or V tile
constexpr int kRing = 4;                      // operand fragments in flight per wave (divides 32)
constexpr int kDist = kRing - 1;              // a fragment is read this many matrix instructions early
constexpr float kRescaleSlack = 8.f;          // log2 units

struct TileRef {
  int start, len;
  bool causal, self;
};

// NW wavefronts per workgroup, each owning one 32-row block; SL: steps between the issue of a
// tile's loads and the barrier that publishes them; SELF: the lists may name tiles of the
// call's own K/V (query prefill) besides pool tiles (pre-encode lists name pool tiles only).
// Row block g = wave covers query head (blockIdx.x * heads_per_block + g / spb) and tokens
// q_start + (g % spb)*32 .. +31, spb = block_m / 32.
// ROPE (query prefill only): Q is un-rotated; the keys carry the rotation of the id they were
// encoded with, and every list entry names the id at which its rows must be rotated instead
// (AttnParams::list_shift: the new in-order positions of Sec. 2.2 as a rotation of the query).
// Entries of one segment share that id, so the Q fragments are rebuilt at segment changes only.
template <int NW, int SL, bool SELF, bool ROPE = false>
__global__ __launch_bounds__(NW * 64, 2) void attn_prefill_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  constexpr int kBlocksPerWave = 16 / NW;  // 1-KiB load blocks of one operand per wave (NW <= 8 < 16)
  constexpr int KS = 2 + SL, VS = 1 + SL;  // LDS stages of K and of V
  static_assert(NW == 1 || NW == 2 || NW == 4 || NW == 8, "wave count");
  static_assert(SL == 1 || SL == 2, "load slack");
  static_assert(32 % kRing == 0 && kDist >= 1 && kDist <= 8, "ring size");
  const unsigned lds0 = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_byte*)smem));

  const int tid = threadIdx.x, lane = tid % 64, l32 = lane % 32, half = lane / 32;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int r = p.n_q_heads / p.n_kv_heads;

  // ---- rows of this wave, tiles of this workgroup ----
  // blockIdx.x = head block, blockIdx.y = position in the launch order: workgroups are handed
  // to the 8 XCDs round-robin by linear id, so with a multiple of 8 head blocks an XCD keeps
  // the same KV heads and meets the Q tiles of one owner back to back (their KV stays in its L2)
  const int tile = __builtin_amdgcn_readfirstlane(p.order[blockIdx.y]);
  const int q_start = __builtin_amdgcn_readfirstlane(p.qtile_tab[tile * 4 + 0]);
  const int q_len = __builtin_amdgcn_readfirstlane(p.qtile_tab[tile * 4 + 1]);
  const int spb = p.block_m / 32;
  const int head = blockIdx.x * p.heads_per_block + wave / spb;
  const int row_local = (wave % spb) * 32 + l32;
  const bool row_valid = row_local < q_len;
  const int row_tok = q_start + min(row_local, q_len - 1);
  const int q_pos = q_start + row_local;
  const int hk = (blockIdx.x * p.heads_per_block) / r;
  // gridDim.z > 1: the list is cut into gridDim.z runs of entries, one workgroup each, whose
  // un-normalised results a second kernel merges (launches with fewer Q tiles than the chip has
  // room for workgroups)
  int e0 = __builtin_amdgcn_readfirstlane(static_cast<int>(p.list_ptr[tile]));
  int n_tiles = __builtin_amdgcn_readfirstlane(static_cast<int>(p.list_ptr[tile + 1])) - e0;
  if (gridDim.z > 1) {
    const int lo = static_cast<int>(static_cast<int64_t>(n_tiles) * blockIdx.z / gridDim.z);
    const int hi = static_cast<int>(static_cast<int64_t>(n_tiles) * (blockIdx.z + 1) / gridDim.z);
    e0 += lo;
    n_tiles = hi - lo;
  }
  if (n_tiles == 0) return;  // cannot happen: every row sees itself, and the host only cuts lists into non-empty runs
  const const_words ent = (const_words)(reinterpret_cast<uintptr_t>(p.list_ent + 2 * static_cast<int64_t>(e0)));

  // byte addresses of this KV head's first token
  const uint64_t kpool = uniform64(reinterpret_cast<uint64_t>(static_cast<const __bf16*>(p.k_pool.ptr) + hk * p.k_pool.stride_head));
  const uint64_t vpool = uniform64(reinterpret_cast<uint64_t>(static_cast<const __bf16*>(p.v_pool.ptr) + hk * p.v_pool.stride_head));
  const uint64_t kself = uniform64(reinterpret_cast<uint64_t>(static_cast<const __bf16*>(p.k_self.ptr) + hk * p.k_self.stride_head));
  const uint64_t vself = uniform64(reinterpret_cast<uint64_t>(static_cast<const __bf16*>(p.v_self.ptr) + hk * p.v_self.stride_head));
  const int kp_stride = static_cast<int>(p.k_pool.stride_tok), vp_stride = static_cast<int>(p.v_pool.stride_tok);
  const int ks_stride = static_cast<int>(p.k_self.stride_tok), vs_stride = static_cast<int>(p.v_self.stride_tok);

  // list entry `it` of this Q tile (scalar loads: the lists are never written while a kernel runs)
  auto tile_ref = [&](int it) DBSA_INLINE {
    const int w0 = ent[2 * it], w1 = ent[2 * it + 1];
    return TileRef{w0, w1 & 0xFFFF, ((w1 >> 16) & 1) != 0, SELF && ((w1 >> 17) & 1) != 0};
  };

  // ---- global -> LDS loads: this wave fills blocks wave*kBlocksPerWave .. of each operand ----
  // lane -> (row, slot) inside block b: row = 4*b + lane/16, slot = lane%16; the piece
  // fetched into that slot is column (slot ^ swizzle(row)).  The byte offsets of a full
  // pool tile only depend on the lane, so they are computed once.
  unsigned k_lane_off[kBlocksPerWave], v_lane_off[kBlocksPerWave];
#pragma unroll
  for (int j = 0; j < kBlocksPerWave; ++j) {
    const int row_in = 4 * (wave * kBlocksPerWave + j) + lane / 16;
    k_lane_off[j] = static_cast<unsigned>(row_in * kp_stride + (((lane % 16) ^ (row_in % 16)) * 8)) * 2u;
    v_lane_off[j] = static_cast<unsigned>(row_in * vp_stride + (((lane % 16) ^ (4 * (row_in % 4))) * 8)) * 2u;
  }
  // this wave's share (kBlocksPerWave 1-KiB blocks) of a K / V tile.  ONE branch per tile picks
  // the full-pool-tile path, whose per-lane offsets are precomputed: decided per block, the
  // branches and their scalar bookkeeping cost more issue time than the loads themselves.
  auto issue_k = [&](const TileRef& t, int stage) DBSA_INLINE {
    const uint64_t base = (t.self ? kself : kpool) + static_cast<uint64_t>(static_cast<unsigned>(t.start)) *
                                                         static_cast<unsigned>(2 * (t.self ? ks_stride : kp_stride));
    const unsigned dst = lds0 + stage * kTileBytes + wave * kBlocksPerWave * 1024;
    if (__builtin_expect(!t.self && t.len == kBN, 1)) {
#pragma unroll
      for (int j = 0; j < kBlocksPerWave; ++j) dma16(base, k_lane_off[j], dst + j * 1024);
    } else {
      const int stride = t.self ? ks_stride : kp_stride;
#pragma unroll
      for (int j = 0; j < kBlocksPerWave; ++j) {
        const int row_in = 4 * (wave * kBlocksPerWave + j) + lane / 16;
        const int row = min(row_in, t.len - 1);  // rows past the tail repeat the last key
        dma16(base, static_cast<unsigned>(row * stride + (((lane % 16) ^ (row_in % 16)) * 8)) * 2u, dst + j * 1024);
      }
    }
  };
  auto issue_v = [&](const TileRef& t, int stage) DBSA_INLINE {
    const uint64_t base = (t.self ? vself : vpool) + static_cast<uint64_t>(static_cast<unsigned>(t.start)) *
                                                         static_cast<unsigned>(2 * (t.self ? vs_stride : vp_stride));
    const unsigned dst = lds0 + (KS + stage) * kTileBytes + wave * kBlocksPerWave * 1024;
    if (__builtin_expect(!t.self && t.len == kBN, 1)) {
#pragma unroll
      for (int j = 0; j < kBlocksPerWave; ++j) dma16(base, v_lane_off[j], dst + j * 1024);
    } else {
      const int stride = t.self ? vs_stride : vp_stride;
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
  // K fragment (kb, c): row kb*32 + l32, slot (2c + half) ^ (l32 % 16)
  // = k_base ^ (32*c): the chunk index only flips bits 5..7 of the swizzled slot offset
  const int k_base = l32 * kRowBytes + ((half ^ (l32 % 16)) * 16);
  // V transpose-read fragment (ob, keys k0..): row k0 + 4*half + j, j = (lane%16)/4; channel
  // slot 4*ob + 2*(l32/16) + (lane%4)/2, swizzled by 4*j; 8-byte half (lane%2)
  // = v_base ^ (64*ob): the channel block only flips bits 6..7 of the swizzled slot offset
  const int v_base = (4 * half + (lane % 16) / 4) * kRowBytes +
                     (((2 * (l32 / 16) + (lane % 4) / 2) ^ (4 * ((lane % 16) / 4))) * 16) + (lane % 2) * 8;
  int kaddr[8], vaddr[4];  // of the K stage / V stage the fragment reads currently walk
#pragma unroll
  for (int c = 0; c < 8; ++c) kaddr[c] = static_cast<int>(lds0) + (k_base ^ (32 * c));
#pragma unroll
  for (int ob = 0; ob < 4; ++ob) vaddr[ob] = static_cast<int>(lds0) + KS * kTileBytes + (v_base ^ (64 * ob));
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

  // ---- Q^T fragments, pre-multiplied by scale*log2(e) ----
  const float c2 = p.scale_log2e;
  bf16x8 qf[kD / 16];
  const const_words lshift = (const_words)(reinterpret_cast<uintptr_t>(p.list_shift + (ROPE ? e0 : 0)));
  // rebuilds qf rotated at id shift + (row inside the tile)
  auto load_q_rotated = [&](int shift) DBSA_INLINE {
    const __bf16* qp = static_cast<const __bf16*>(p.q.ptr) + static_cast<int64_t>(row_tok) * p.q.stride_tok +
                       static_cast<int64_t>(head) * p.q.stride_head + 8 * half;
    const int id = min(max(shift + row_local, 0), p.rope_n_pos - 1);
    const float* rot = p.rope_table + static_cast<int64_t>(id) * kD + 16 * half;
    load_query_fragments<true>(qp, rot, c2, qf);
  };
  int cur_shift = 0, nxt_shift = 0;  // rotation ids of the entry whose scores are computed next / after that
  if constexpr (ROPE) {
    cur_shift = lshift[0];
    nxt_shift = n_tiles > 1 ? lshift[1] : cur_shift;
    load_q_rotated(cur_shift);
  } else {
    const __bf16* qp = static_cast<const __bf16*>(p.q.ptr) + static_cast<int64_t>(row_tok) * p.q.stride_tok +
                       static_cast<int64_t>(head) * p.q.stride_head + 8 * half;
    load_query_fragments<false>(qp, nullptr, c2, qf);
  }

  floatx16 o[kD / 32];
  float m_run = 0.f, l_run = 0.f;  // running max (log2 domain), this lane's share of the row sum
#pragma unroll
  for (int ob = 0; ob < kD / 32; ++ob)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[ob][i] = 0.f;

  // masks of a causal or short tile, applied to the scores
  auto apply_mask = [&](floatx16 (&s)[2], const TileRef& t) DBSA_INLINE {
    const int limit = t.causal ? (q_pos - t.start) : kBN;  // visible iff key_local <= limit
    int key0 = 4 * half;
    asm volatile("" : "+v"(key0));  // keeps 32 loop-invariant key indices out of registers: this path is rare
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key_local = key0 + (kb * 32 + 8 * (i / 4) + (i % 4));
        const bool vis = key_local < t.len && key_local <= limit;
        s[kb][i] = vis ? s[kb][i] : -INFINITY;
      }
  };

  // ---- prologue: K(0 .. 1+SL), V(0 .. SL-1) in flight; scores of tile 0 fix the first running max ----
  // refs[i] = list entry it+1+i at the top of step it (i = 0 .. SL+1; zero length past the end)
  TileRef cur = tile_ref(0), refs[2 + SL];
#pragma unroll
  for (int i = 0; i < 2 + SL; ++i) refs[i] = (i + 1 < n_tiles) ? tile_ref(i + 1) : TileRef{0, 0, false, false};
  issue_k(cur, 0);
#pragma unroll
  for (int i = 0; i < 1 + SL; ++i)
    if (i + 1 < n_tiles) issue_k(refs[i], i + 1);
  issue_v(cur, 0);
  if (SL == 2 && n_tiles > 1) issue_v(refs[0], 1);
  wait_vmcnt<0>();
  __syncthreads();

  floatx16 s_a[2], s_b[2];  // scores (minus running max) of the tile being consumed / of the next tile
  float mx_cur;             // row maximum of the tile being consumed, relative to the running max
#pragma unroll
  for (int kb = 0; kb < 2; ++kb)
#pragma unroll
    for (int i = 0; i < 16; ++i) s_a[kb][i] = 0.f;
  static_for<16>([&](auto T) DBSA_INLINE {
    constexpr int t = decltype(T)::value;
    const bf16x8 kf = ld_k(T);
    s_a[t / 8] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t % 8], s_a[t / 8], 0, 0, 0);
  });
  if (cur.causal || cur.len < kBN) apply_mask(s_a, cur);
  {
    float m = s_a[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) m = fmaxf(m, s_a[kb][i]);
    // every row sees at least one key of its first listed tile, so the maximum is finite
    m_run = fmaxf(half_swap_max(m), -1.0e30f);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s_a[kb][i] -= m_run;
    mx_cur = 0.f;
  }
  // minus the running maximum in every element: the C operand of the first matrix instruction of
  // each score block, so that accumulators need no per-step initialisation
  floatx16 neg_m;
#pragma unroll
  for (int i = 0; i < 16; ++i) neg_m[i] = -m_run;

  // the fragment reads now walk K stage 1 (tile 1) and V stage 0 (tile 0); the first kDist
  // fragments of K(1) enter the ring (stale data if the list has one entry: never used)
  int k_rd = 1, v_rd = 0;    // stage the K / V fragment addresses point into
  int k_wr = 0, v_wr = SL;   // stage the loads issued in step 0 fill: K(2+SL) -> (2+SL) % KS, V(SL)
#pragma unroll
  for (int c = 0; c < 8; ++c) kaddr[c] += kTileBytes;
  bf16x8 ring[kRing];
  static_for<kDist>([&](auto T) DBSA_INLINE { ring[decltype(T)::value % kRing] = ld_k(T); });

  // One tile step.  On entry s_cur holds the (masked) scores of tile `it` minus m_run, mx_cur
  // their row maximum, neg_m minus m_run in every element, and the ring the first kDist
  // fragments of K(it+1).  K(it+1) is visible since the previous barrier; V(it) becomes
  // visible with this one.  The last tile computes an s_nxt nobody uses (stale LDS contents)
  // so that every tile runs the same straight-line code.
  auto tile_step = [&](int it, floatx16 (&s_cur)[2], floatx16 (&s_nxt)[2]) DBSA_INLINE {
    // what this step needs was issued SL steps ago; with SL == 2 the K and V loads of the
    // previous step (2*kBlocksPerWave instructions, if that step issued both sets) may stay in flight
    if (SL == 2 && it + 1 + SL < n_tiles)
      wait_vmcnt<(SL == 2 ? 2 * kBlocksPerWave : 0)>();
    else
      wait_vmcnt<0>();
    __syncthreads();

    // rare: some row's maximum outgrew the lagging running maximum
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(mx_cur > kRescaleSlack) != 0, 0)) {
      const float delta = fmaxf(mx_cur, 0.f);
      const float alpha = __builtin_amdgcn_exp2f(-delta);
      m_run += delta;
      l_run *= alpha;
#pragma unroll
      for (int ob = 0; ob < kD / 32; ++ob) o[ob] *= alpha;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) s_cur[kb][i] -= delta;
#pragma unroll
      for (int i = 0; i < 16; ++i) neg_m[i] -= delta;
    }

    if constexpr (ROPE) {
      // this step computes the scores of entry it+1: rebuild Q when that entry starts a new segment
      if (__builtin_expect(nxt_shift != cur_shift, 0)) {
        cur_shift = nxt_shift;
        load_q_rotated(cur_shift);
      }
    }
    const bool has_next = it + 1 < n_tiles;
    const TileRef nxt = refs[0];
    // List entry it+3+SL (zero past the end), needed by the next step's K load.  Requested FIRST:
    // a scalar load shares its counter with the LDS fragment reads and returns out of order with
    // them, so while it is in flight every fragment wait drains the whole queue; behind the
    // load instructions of this step it has returned before the first such wait.
    int in_w0 = 0, in_w1 = 0;
    if (it + 3 + SL < n_tiles) {
      in_w0 = ent[2 * (it + 3 + SL)];
      in_w1 = ent[2 * (it + 3 + SL) + 1];
    }
    if constexpr (ROPE) {
      if (it + 2 < n_tiles) nxt_shift = lshift[it + 2];
    }
    bf16x2 pk[2][8];
    float p0 = 0.f, p1 = 0.f;  // exponentials of one matrix step, packed during the next

    // -- S(it+1) = K(it+1) Q^T (matrix pipe) || probabilities of tile it (vector ALU) --
    __builtin_amdgcn_sched_barrier(0);
    static_for<16>([&](auto T) DBSA_INLINE {
      constexpr int t = decltype(T)::value;
      s_nxt[t / 8] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[t % kRing], qf[t % 8], t % 8 == 0 ? neg_m : s_nxt[t / 8],
                                                             0, 0, 0);
      if constexpr (t + kDist < 16)
        ring[(t + kDist) % kRing] = ld_k(std::integral_constant<int, (t + kDist) % 16>{});
      else
        ring[(t + kDist) % kRing] = ld_v(std::integral_constant<int, (t + kDist) % 16>{});
      if constexpr (t == 0) {
        // this step's loads go out behind the first matrix instruction: K(it+2+SL), V(it+SL).
        // (Spreading them over the phase, one per few matrix instructions, measured slower: every
        // load sits behind a branch on the list length, and each branch splits the straight-line code.)
        if (it + 2 + SL < n_tiles) issue_k(refs[1 + SL], k_wr);
        if (it + SL < n_tiles) issue_v(refs[SL - 1], v_wr);
      }
      if constexpr (t > 0) {
        constexpr int u = t - 1;
        pk[u / 8][u % 8] = __builtin_convertvector(floatx2{p0, p1}, bf16x2);
        l_run += p0 + p1;
        asm volatile("" : "+v"(pk[u / 8][u % 8]));
      }
      p0 = __builtin_amdgcn_exp2f(s_cur[t / 8][2 * (t % 8)]);
      p1 = __builtin_amdgcn_exp2f(s_cur[t / 8][2 * (t % 8) + 1]);
      // keep the vector work in this step, next to the MFMA it overlaps with
      asm volatile("" : "+v"(p0), "+v"(p1), "+v"(l_run));
      __builtin_amdgcn_sched_barrier(0);
    });
    pk[1][7] = __builtin_convertvector(floatx2{p0, p1}, bf16x2);
    l_run += p0 + p1;
    if (__builtin_expect(has_next && (nxt.causal || nxt.len < kBN), 0)) apply_mask(s_nxt, nxt);
    {
      // every K fragment of tile it+1 has been requested: the K addresses move on to the stage of K(it+2)
      const int k_next = (k_rd + 1 == KS) ? 0 : k_rd + 1;
      const int dk = (k_next - k_rd) * kTileBytes;
#pragma unroll
      for (int c = 0; c < 8; ++c) kaddr[c] += dk;
      k_rd = k_next;
    }

    // -- O^T += V(it)^T P^T (matrix pipe) || row maximum of tile it+1, next accumulator init (vector ALU) --
    float mt = s_nxt[0][0];
    __builtin_amdgcn_sched_barrier(0);
    static_for<16>([&](auto T) DBSA_INLINE {
      constexpr int t = decltype(T)::value;
      union {
        bf16x8 v;
        bf16x2 p2[4];
      } pf;
#pragma unroll
      for (int e = 0; e < 4; ++e) pf.p2[e] = pk[t / 8][4 * ((t / 4) % 2) + e];
      o[t % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[(16 + t) % kRing], pf.v, o[t % 4], 0, 0, 0);
      if constexpr (t + kDist < 16)
        ring[(16 + t + kDist) % kRing] = ld_v(std::integral_constant<int, (t + kDist) % 16>{});
      else
        ring[(16 + t + kDist) % kRing] = ld_k(std::integral_constant<int, (t + kDist) % 16>{});
      mt = fmaxf(mt, fmaxf(s_nxt[t / 8][2 * (t % 8)], s_nxt[t / 8][2 * (t % 8) + 1]));
      asm volatile("" : "+v"(mt));
      __builtin_amdgcn_sched_barrier(0);
    });
    mx_cur = half_swap_max(mt);

    // bookkeeping for the next step
    {
      const int v_next = (v_rd + 1 == VS) ? 0 : v_rd + 1;
      const int dv = (v_next - v_rd) * kTileBytes;
#pragma unroll
      for (int ob = 0; ob < 4; ++ob) vaddr[ob] += dv;
      v_rd = v_next;
      k_wr = (k_wr + 1 == KS) ? 0 : k_wr + 1;
      v_wr = (v_wr + 1 == VS) ? 0 : v_wr + 1;
#pragma unroll
      for (int i = 0; i < 1 + SL; ++i) refs[i] = refs[i + 1];
      refs[1 + SL] = TileRef{in_w0, in_w1 & 0xFFFF, ((in_w1 >> 16) & 1) != 0, SELF && ((in_w1 >> 17) & 1) != 0};
    }
  };

  for (int it = 0; it < n_tiles; it += 2) {
    tile_step(it, s_a, s_b);
    if (it + 1 >= n_tiles) break;
    tile_step(it + 1, s_b, s_a);
  }

  // ---- epilogue ----
  {
    const float l_tot = half_swap_sum(l_run);
    if (!row_valid) return;
    if (gridDim.z > 1) {
      float* part = p.partial + ((static_cast<int64_t>(row_tok) * p.n_q_heads + head) * gridDim.z + blockIdx.z) *
                                    (kD + kPartialPad);
#pragma unroll
      for (int ob = 0; ob < kD / 32; ++ob)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<floatx4*>(part + 32 * ob + 8 * g + 4 * half) =
              floatx4{o[ob][4 * g], o[ob][4 * g + 1], o[ob][4 * g + 2], o[ob][4 * g + 3]};
      if (half == 0) {
        part[kD] = m_run;
        part[kD + 1] = l_tot;
      }
      return;
    }
    const float inv = 1.f / l_tot;
    __bf16* op = static_cast<__bf16*>(const_cast<void*>(p.o.ptr)) + static_cast<int64_t>(row_tok) * p.o.stride_tok +
                 static_cast<int64_t>(head) * p.o.stride_head + 4 * half;
#pragma unroll
    for (int ob = 0; ob < kD / 32; ++ob)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        union {
          bf16x4 v;
          bf16x2 p2[2];
        } w;
        w.p2[0] = __builtin_convertvector(floatx2{o[ob][4 * g] * inv, o[ob][4 * g + 1] * inv}, bf16x2);
        w.p2[1] = __builtin_convertvector(floatx2{o[ob][4 * g + 2] * inv, o[ob][4 * g + 3] * inv}, bf16x2);
        *reinterpret_cast<bf16x4*>(op + 32 * ob + 8 * g) = w.v;
      }
    if (p.lse && half == 0)
      p.lse[static_cast<int64_t>(head) * p.lse_stride + row_tok] = (m_run + __log2f(l_tot)) * 0.69314718055994531f;
  }
}

// Merge of the n_split partial states of a (row, head): 32 threads per pair, four channels each.
// o = sum_z 2^(m_z - m*) acc_z / sum_z 2^(m_z - m*) l_z, statistics in the log2 domain.
constexpr int kMergePairs = 8;  // (row, head) pairs per workgroup of 256 threads
__global__ __launch_bounds__(32 * kMergePairs) void prefill_merge_kernel(AttnParams p, int n_rows, int n_split) {
  const int64_t pair = static_cast<int64_t>(blockIdx.x) * kMergePairs + threadIdx.x / 32;
  if (pair >= static_cast<int64_t>(n_rows) * p.n_q_heads) return;
  const int row = static_cast<int>(pair / p.n_q_heads), head = static_cast<int>(pair % p.n_q_heads);
  const int d = 4 * (threadIdx.x % 32);
  const float* part = p.partial + pair * n_split * (kD + kPartialPad);
  float m_star = -1.0e30f;
  for (int z = 0; z < n_split; ++z) m_star = fmaxf(m_star, part[z * (kD + kPartialPad) + kD]);
  float l = 0.f;
  floatx4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int z = 0; z < n_split; ++z) {
    const float w = __builtin_amdgcn_exp2f(part[z * (kD + kPartialPad) + kD] - m_star);
    l = fmaf(part[z * (kD + kPartialPad) + kD + 1], w, l);
    acc += *reinterpret_cast<const floatx4*>(part + z * (kD + kPartialPad) + d) * w;
  }
  const float inv = 1.f / l;
  union {
    bf16x4 v;
    bf16x2 p2[2];
  } w;
  w.p2[0] = __builtin_convertvector(floatx2{acc[0] * inv, acc[1] * inv}, bf16x2);
  w.p2[1] = __builtin_convertvector(floatx2{acc[2] * inv, acc[3] * inv}, bf16x2);
  __bf16* o = static_cast<__bf16*>(const_cast<void*>(p.o.ptr));
  *reinterpret_cast<bf16x4*>(o + static_cast<int64_t>(row) * p.o.stride_tok + static_cast<int64_t>(head) * p.o.stride_head + d) = w.v;
  if (p.lse && d == 0) p.lse[static_cast<int64_t>(head) * p.lse_stride + row] = (m_star + __log2f(l)) * 0.69314718055994531f;
}

template <int NW, int SL, bool SELF, bool ROPE = false>
hipError_t launch_cfg(const AttnParams& p, hipStream_t stream) {
  constexpr int lds_bytes = (3 + 2 * SL) * kTileBytes;
  static std::atomic<bool> attr_set{false};  // setting it twice from two threads is harmless
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_prefill_kernel<NW, SL, SELF, ROPE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int n_split = p.q_split > 1 ? p.q_split : 1;
  dim3 grid(p.n_q_heads / p.heads_per_block, p.n_qtiles, n_split), block(NW * 64);
  attn_prefill_kernel<NW, SL, SELF, ROPE><<<grid, block, lds_bytes, stream>>>(p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || n_split == 1) return e;
  const int64_t pairs = static_cast<int64_t>(p.n_rows) * p.n_q_heads;
  prefill_merge_kernel<<<dim3(static_cast<unsigned>((pairs + kMergePairs - 1) / kMergePairs)), dim3(32 * kMergePairs), 0,
                         stream>>>(p, p.n_rows, n_split);
  return hipGetLastError();
}

template <int NW, int SL>
hipError_t launch_stage(const AttnParams& p, hipStream_t stream) {
  if (p.rope_table) return p.query_stage ? launch_cfg<NW, SL, true, true>(p, stream) : hipErrorInvalidValue;
  return p.query_stage ? launch_cfg<NW, SL, true>(p, stream) : launch_cfg<NW, SL, false>(p, stream);
}

}  // namespace

// One workgroup takes heads_per_block * (block_m / 32) row blocks of 32 rows, one per wave.  Eight
// waves fill a compute unit on their own (one workgroup per CU: 112 KiB of LDS buy two steps of
// load slack); smaller workgroups share a CU in pairs and take 80 KiB each.
hipError_t launch_prefill_pipelined(const AttnParams& p, hipStream_t stream) {
  if (p.n_qtiles == 0) return hipSuccess;
  const int row_blocks = p.heads_per_block * (p.block_m / 32);
  // four or eight row blocks: the kernel with 64 rows per wave, one wave per SIMD (persistent if
  // the call carries a schedule, else one workgroup per Q tile and run)
  if (row_blocks == 4 || row_blocks == 8) {
    hipError_t e = launch_prefill64(p, stream);
    const int n_split = p.q_split > 1 ? p.q_split : 1;
    if (e != hipSuccess || n_split == 1) return e;
    const int64_t pairs = static_cast<int64_t>(p.n_rows) * p.n_q_heads;
    prefill_merge_kernel<<<dim3(static_cast<unsigned>((pairs + kMergePairs - 1) / kMergePairs)), dim3(32 * kMergePairs), 0,
                           stream>>>(p, p.n_rows, n_split);
    return hipGetLastError();
  }
  switch (row_blocks) {
    case 1: return launch_stage<1, 1>(p, stream);
    case 2: return launch_stage<2, 1>(p, stream);
    case 4: return launch_stage<4, 1>(p, stream);
    case 8: return launch_stage<8, 2>(p, stream);
    default: return hipErrorInvalidValue;
  }
}
