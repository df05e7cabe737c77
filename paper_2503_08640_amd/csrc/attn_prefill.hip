// Software-pipelined bf16 MFMA attention for prefill-shaped calls (pre-encode, Sec. 2.1;
// query prefill, Sec. 2.2) at head_dim 128 on gfx950.  Same mathematics and register
// plan as attn_mfma.hip (transposed scores S^T = K Q^T, per-lane softmax statistics,
// O^T = V^T P^T).  Measured on MI355X, one wavefront issues at most one instruction every
// ~8 cycles and two wavefronts per SIMD fit the register budget, so the kernel is built
// around a small instruction count per MFMA:
//
//   * K and V tiles go from global memory straight into LDS with
//     global_load_lds_dwordx4 (no staging registers, no ds_write).  A wave-level load
//     fills 1 KiB of LDS in lane order, so the layout is unpadded and bank conflicts are
//     avoided by choosing WHICH 16-byte piece each lane fetches: row-major 256-byte rows
//     whose 16-byte slots are XOR-swizzled, K by (row % 16) for the 128-bit fragment
//     reads (16 consecutive rows, same slot -> 16 distinct bank groups) and V by
//     4*(row % 4) for the 64-bit transpose reads (4 rows x 4 slots per half-wave).
//   * two LDS stages per operand and ONE workgroup barrier per KV tile: while tile j is
//     being consumed, K of tile j+2 and V of tile j+1 are in flight.
//   * Q is pre-multiplied by scale*log2(e) when its fragments are loaded, and the score
//     accumulators start at minus the running row maximum, so that a probability is one
//     v_exp_f32 of the MFMA result; the row sum comes from a packed bf16 dot product of
//     the rounded probabilities with ones.
//   * the scores of tile j+1 are issued in the same straight-line steps as the
//     exponentials of tile j, and the row maxima of tile j+1 in the same steps as the
//     second product of tile j, with K/V fragments fetched two steps ahead.
//   * the running maximum may lag the true maximum by kRescaleSlack (weights then reach
//     2^slack at most, harmless in fp32/bf16): accumulators are rescaled only when some
//     row of the wave outgrows it, which is rare once a few tiles have been seen.
#include <cstdint>

#include "kernels.hpp"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
constexpr int kBN = 64;                       // keys per KV tile
constexpr int kRowBytes = kD * 2;             // 256
constexpr int kTileBytes = kBN * kRowBytes;   // 16 KiB per K or V tile
constexpr int kLdsBytes = 4 * kTileBytes;     // K stage 0/1, V stage 0/1
constexpr float kRescaleSlack = 8.f;          // log2 units

typedef __attribute__((address_space(3))) unsigned char lds_byte;

__device__ inline bf16x4 lds_read_tr(const lds_byte* p) {
  typedef __attribute__((address_space(3))) shortx4* tr_ptr;
  const shortx4 t = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(p));
  return __builtin_bit_cast(bf16x4, t);
}

// Combine a value held by lanes l and l^32 (the two half-waves hold the two key halves of
// the same row).
__device__ inline float half_swap_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float half_swap_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 16 bytes per lane from global memory straight into LDS: lane l's piece lands at
// dst + 16*l.  Issued through inline assembly so that the transfer stays asynchronous:
// the kernel waits for it explicitly (vmcnt) right before the workgroup barrier that
// publishes the stage, instead of before the next LDS read of any stage.
__device__ inline void dma16(const void* gbase_in, unsigned byte_off, lds_byte* dst) {
  // both addresses are wave-uniform by construction; say so to the compiler, which must
  // place them in scalar registers
  const uint64_t g = reinterpret_cast<uint64_t>(gbase_in);
  // (readfirstlane returns a signed int: widen through unsigned, or the low word would be sign-extended)
  const unsigned g_hi = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(g >> 32)));
  const unsigned g_lo = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(g & 0xFFFFFFFFu)));
  const void* gbase = reinterpret_cast<const void*>((static_cast<uint64_t>(g_hi) << 32) | static_cast<uint64_t>(g_lo));
  const unsigned m0v = static_cast<unsigned>(
      __builtin_amdgcn_readfirstlane(static_cast<int>(reinterpret_cast<uintptr_t>(dst) & 0xFFFFFFFFu)));
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(m0v), "v"(byte_off), "s"(gbase)
               : "memory");
}

struct TileRef {
  int start, len;
  bool causal, self;
};

// NW wavefronts per workgroup, RB 32-row blocks per wavefront; SELF: the lists may name tiles of
// the call's own K/V (query prefill) besides pool tiles (pre-encode lists name pool tiles only).
// Row block g = wave*RB + rb
// covers query head (blockIdx.x * heads_per_block + g / spb) and tokens
// q_start + (g % spb)*32 .. +31, spb = block_m / 32.
template <int NW, int RB, bool SELF>
__global__ __launch_bounds__(NW * 64, 2) void attn_prefill_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  constexpr int kBlocksPerWave = 16 / NW;  // 1-KiB load blocks of one operand per wave (NW <= 8 < 16)
  static_assert(NW == 1 || NW == 2 || NW == 4 || NW == 8, "wave count");
  lds_byte* lds = (lds_byte*)smem;

  const int tid = threadIdx.x, lane = tid % 64, l32 = lane % 32, half = lane / 32;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int r = p.n_q_heads / p.n_kv_heads;

  // ---- rows of this wave, tiles of this workgroup ----
  // (loaded through vector memory; readfirstlane moves the wave-uniform values to scalar registers)
  // blockIdx.x = head block, blockIdx.y = position in the launch order: workgroups are handed
  // to the 8 XCDs round-robin by linear id, so with a multiple of 8 head blocks an XCD keeps
  // the same KV heads and meets the Q tiles of one owner back to back (their KV stays in its L2)
  const int tile = __builtin_amdgcn_readfirstlane(p.order[blockIdx.y]);
  const int q_start = __builtin_amdgcn_readfirstlane(p.qtile_tab[tile * 4 + 0]);
  const int q_len = __builtin_amdgcn_readfirstlane(p.qtile_tab[tile * 4 + 1]);
  const int spb = p.block_m / 32;
  int head[RB], row_tok[RB], q_pos[RB];
  bool row_valid[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int g = wave * RB + rb;
    const int sub = g % spb;
    head[rb] = blockIdx.x * p.heads_per_block + g / spb;
    const int row_local = sub * 32 + l32;
    row_valid[rb] = row_local < q_len;
    row_tok[rb] = q_start + min(row_local, q_len - 1);
    q_pos[rb] = q_start + row_local;
  }
  const int hk = (blockIdx.x * p.heads_per_block) / r;
  const int e0 = __builtin_amdgcn_readfirstlane(static_cast<int>(p.list_ptr[tile]));
  const int n_tiles = __builtin_amdgcn_readfirstlane(static_cast<int>(p.list_ptr[tile + 1])) - e0;
  const int32_t* ent = p.list_ent + 2 * static_cast<int64_t>(e0);
  if (n_tiles == 0) return;  // cannot happen for a well-formed layout: every row sees itself

  const __bf16* kpool = static_cast<const __bf16*>(p.k_pool.ptr) + hk * p.k_pool.stride_head;
  const __bf16* vpool = static_cast<const __bf16*>(p.v_pool.ptr) + hk * p.v_pool.stride_head;
  const __bf16* kself = static_cast<const __bf16*>(p.k_self.ptr) + hk * p.k_self.stride_head;
  const __bf16* vself = static_cast<const __bf16*>(p.v_self.ptr) + hk * p.v_self.stride_head;
  const int kp_stride = static_cast<int>(p.k_pool.stride_tok), vp_stride = static_cast<int>(p.v_pool.stride_tok);
  const int ks_stride = static_cast<int>(p.k_self.stride_tok), vs_stride = static_cast<int>(p.v_self.stride_tok);

  auto tile_ref = [&](int it) {
    const int w0 = __builtin_amdgcn_readfirstlane(ent[2 * it]), w1 = __builtin_amdgcn_readfirstlane(ent[2 * it + 1]);
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
  auto issue_k = [&](const TileRef& t, int stage) {
    const __bf16* base = (t.self ? kself : kpool) + static_cast<int64_t>(t.start) * (t.self ? ks_stride : kp_stride);
    lds_byte* dst = lds + stage * kTileBytes + wave * kBlocksPerWave * 1024;
    if (!t.self && t.len == kBN) {
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
  auto issue_v = [&](const TileRef& t, int stage) {
    const __bf16* base = (t.self ? vself : vpool) + static_cast<int64_t>(t.start) * (t.self ? vs_stride : vp_stride);
    lds_byte* dst = lds + (2 + stage) * kTileBytes + wave * kBlocksPerWave * 1024;
    if (!t.self && t.len == kBN) {
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

  // ---- per-lane LDS read addresses (bytes, inside a tile) ----
  // K fragment (kb, c): row kb*32 + l32, slot (2c + half) ^ (l32 % 16)
  // = k_base ^ (32*c): the chunk index only flips bits 5..7 of the swizzled slot offset
  const int k_base = l32 * kRowBytes + ((half ^ (l32 % 16)) * 16);
  // V transpose-read fragment (ob, keys k0..): row k0 + 4*half + j, j = (lane%16)/4; channel
  // slot 4*ob + 2*(l32/16) + (lane%4)/2, swizzled by 4*j; 8-byte half (lane%2)
  // = v_base ^ (64*ob): the channel block only flips bits 6..7 of the swizzled slot offset
  const int v_base = (4 * half + (lane % 16) / 4) * kRowBytes +
                     (((2 * (l32 / 16) + (lane % 4) / 2) ^ (4 * ((lane % 16) / 4))) * 16) + (lane % 2) * 8;

  // ---- Q^T fragments, pre-multiplied by scale*log2(e) ----
  const float c2 = p.scale_log2e;
  bf16x8 qf[RB][kD / 16];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const __bf16* qp = static_cast<const __bf16*>(p.q.ptr) + static_cast<int64_t>(row_tok[rb]) * p.q.stride_tok +
                       static_cast<int64_t>(head[rb]) * p.q.stride_head + 8 * half;
#pragma unroll
    for (int c = 0; c < kD / 16; ++c) {
      const bf16x8 raw = *reinterpret_cast<const bf16x8*>(qp + 16 * c);
      union {
        bf16x8 v;
        bf16x2 p2[4];
      } sc;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        sc.p2[e] = __builtin_convertvector(
            floatx2{static_cast<float>(raw[2 * e]) * c2, static_cast<float>(raw[2 * e + 1]) * c2}, bf16x2);
      qf[rb][c] = sc.v;
    }
  }

  floatx16 o[RB][kD / 32];
  float m_run[RB], l_run[RB];  // running max (log2 domain), this lane's share of the row sum
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    m_run[rb] = 0.f;
    l_run[rb] = 0.f;
#pragma unroll
    for (int ob = 0; ob < kD / 32; ++ob)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[rb][ob][i] = 0.f;
  }

  // ---- building blocks of one tile step -------------------------------------------------
  // K fragment t (t = kb*8 + c) of K stage `stage`; V fragment t (t = kb*8 + ch*4 + ob).
  auto ld_k = [&](int stage, int t) {
    return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(
        lds + stage * kTileBytes + (k_base ^ (32 * (t % 8))) + (t / 8) * 32 * kRowBytes);
  };
  auto ld_v = [&](int stage, int t) {
    const lds_byte* vp =
        lds + (2 + stage) * kTileBytes + (v_base ^ (64 * (t % 4))) + ((t / 8) * 32 + ((t / 4) % 2) * 16) * kRowBytes;
    const bf16x4 lo = lds_read_tr(vp);
    const bf16x4 hi = lds_read_tr(vp + 8 * kRowBytes);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  };
  // masks of a causal or short tile, applied to the scores
  auto apply_mask = [&](floatx16 (&s)[RB][2], const TileRef& t) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const int limit = t.causal ? (q_pos[rb] - t.start) : kBN;  // visible iff key_local <= limit
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key_local = kb * 32 + 8 * (i / 4) + 4 * half + (i % 4);
          const bool vis = key_local < t.len && key_local <= limit;
          s[rb][kb][i] = vis ? s[rb][kb][i] : -INFINITY;
        }
    }
  };
  auto row_max = [&](const floatx16 (&s)[RB][2], float (&mx)[RB]) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float m = s[rb][0][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) m = fmaxf(m, s[rb][kb][i]);
      mx[rb] = half_swap_max(m);
    }
  };

  // ---- prologue: K(0), V(0), K(1) in flight; scores of tile 0 fix the first running max ----
  TileRef cur = tile_ref(0), nxt{};
  floatx16 s_a[RB][2], s_b[RB][2];  // scores (minus running max) of the tile being consumed / of the next tile
  float mx_cur[RB];                 // row maxima of the tile being consumed, relative to the running max
  issue_k(cur, 0);
  issue_v(cur, 0);
  if (n_tiles > 1) {
    nxt = tile_ref(1);
    issue_k(nxt, 1);
  }
  __builtin_amdgcn_s_waitcnt(0);  // all counters: own loads have landed
  __syncthreads();
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s_a[rb][kb][i] = 0.f;
#pragma unroll
  for (int t = 0; t < 16; ++t) {
    const bf16x8 kf = ld_k(0, t);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
      s_a[rb][t / 8] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[rb][t % 8], s_a[rb][t / 8], 0, 0, 0);
  }
  if (cur.causal || cur.len < kBN) apply_mask(s_a, cur);
  row_max(s_a, mx_cur);
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    // every row sees at least one key of its first listed tile, so the maximum is finite
    m_run[rb] = fmaxf(mx_cur[rb], -1.0e30f);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s_a[rb][kb][i] -= m_run[rb];
    mx_cur[rb] = 0.f;
  }

  // One tile step.  On entry s_cur holds the (masked) scores of tile `it` minus m_run and
  // mx_cur their row maxima; K(it+1) -> K stage 1-STAGE and V(it) -> V stage STAGE have
  // been issued.  The last tile computes an s_nxt nobody uses (stale LDS contents) so that
  // every tile runs the same straight-line code.
#define DBSA_TILE_STEP(STAGE, s_cur, s_nxt)                                                                      \
  {                                                                                                              \
    __builtin_amdgcn_s_waitcnt(0);                                                                               \
    __syncthreads();                                                                                             \
    /* first fragments of both products right away: their LDS latency hides behind the bookkeeping below */     \
    bf16x8 kf[3], vf[3];                                                                                         \
    kf[0] = ld_k(1 - STAGE, 0);                                                                                  \
    kf[1] = ld_k(1 - STAGE, 1);                                                                                  \
    vf[0] = ld_v(STAGE, 0);                                                                                      \
    vf[1] = ld_v(STAGE, 1);                                                                                      \
    __builtin_amdgcn_sched_barrier(0);                                                                           \
    TileRef nn{};                                                                                                \
    if (it + 2 < n_tiles) {                                                                                      \
      nn = tile_ref(it + 2);                                                                                     \
      issue_k(nn, STAGE);                                                                                        \
    }                                                                                                            \
    const bool has_next = it + 1 < n_tiles;                                                                      \
    if (has_next) issue_v(nxt, 1 - STAGE);                                                                       \
    {                                                                                                            \
      bool grow = false;                                                                                         \
      _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) grow = grow || (mx_cur[rb] > kRescaleSlack);             \
      if (__builtin_amdgcn_ballot_w64(grow) != 0) {                                                              \
        _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) {                                                      \
          const float delta = fmaxf(mx_cur[rb], 0.f);                                                            \
          const float alpha = __builtin_amdgcn_exp2f(-delta);                                                    \
          m_run[rb] += delta;                                                                                    \
          l_run[rb] *= alpha;                                                                                    \
          _Pragma("unroll") for (int ob = 0; ob < kD / 32; ++ob) o[rb][ob] *= alpha;                             \
          _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) _Pragma("unroll") for (int i = 0; i < 16; ++i)        \
              s_cur[rb][kb][i] -= delta;                                                                         \
        }                                                                                                        \
      }                                                                                                          \
    }                                                                                                            \
    /* -- scores of the next tile (matrix pipe) || probabilities of this tile (vector ALU) -- */                \
    bf16x2 pk[RB][2][8];                                                                                         \
    _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) _Pragma("unroll") for (int kb = 0; kb < 2; ++kb)           \
        _Pragma("unroll") for (int i = 0; i < 16; ++i) s_nxt[rb][kb][i] = -m_run[rb];                            \
    {                                                                                                            \
      const bf16x2 ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};                                \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
      _Pragma("unroll") for (int t = 0; t < 16; ++t) {                                                           \
        if (t + 2 < 16) kf[(t + 2) % 3] = ld_k(1 - STAGE, t + 2);                                                \
        _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) s_nxt[rb][t / 8] =                                     \
            __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t % 3], qf[rb][t % 8], s_nxt[rb][t / 8], 0, 0, 0);        \
        _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) {                                                      \
          const int kb = t / 8, i = 2 * (t % 8);                                                                 \
          const float p0 = __builtin_amdgcn_exp2f(s_cur[rb][kb][i]);                                             \
          const float p1 = __builtin_amdgcn_exp2f(s_cur[rb][kb][i + 1]);                                         \
          pk[rb][kb][t % 8] = __builtin_convertvector(floatx2{p0, p1}, bf16x2);                                  \
          /* row sum of the ROUNDED probabilities: the same values the second product uses */                   \
          l_run[rb] = __builtin_amdgcn_fdot2_f32_bf16(pk[rb][kb][t % 8], ones, l_run[rb], false);                \
          /* keep the exponentials in this step, next to the MFMA they overlap with */                          \
          asm volatile("" : "+v"(pk[rb][kb][t % 8]), "+v"(l_run[rb]));                                           \
        }                                                                                                        \
        __builtin_amdgcn_sched_barrier(0);                                                                       \
      }                                                                                                          \
    }                                                                                                            \
    if (has_next && (nxt.causal || nxt.len < kBN)) apply_mask(s_nxt, nxt);                                       \
    /* -- O^T += V^T P^T (matrix pipe) || row maxima of the next tile (vector ALU) -- */                        \
    {                                                                                                            \
      float mt[RB];                                                                                              \
      _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) mt[rb] = s_nxt[rb][0][0];                                \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
      _Pragma("unroll") for (int t = 0; t < 16; ++t) {                                                           \
        if (t + 2 < 16) vf[(t + 2) % 3] = ld_v(STAGE, t + 2);                                                    \
        _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) {                                                      \
          union {                                                                                                \
            bf16x8 v;                                                                                            \
            bf16x2 p2[4];                                                                                        \
          } pf;                                                                                                  \
          _Pragma("unroll") for (int e = 0; e < 4; ++e) pf.p2[e] = pk[rb][t / 8][4 * ((t / 4) % 2) + e];         \
          o[rb][t % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t % 3], pf.v, o[rb][t % 4], 0, 0, 0);        \
          mt[rb] = fmaxf(mt[rb], fmaxf(s_nxt[rb][t / 8][2 * (t % 8)], s_nxt[rb][t / 8][2 * (t % 8) + 1]));       \
          asm volatile("" : "+v"(mt[rb]));                                                                       \
        }                                                                                                        \
        __builtin_amdgcn_sched_barrier(0);                                                                       \
      }                                                                                                          \
      _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) mx_cur[rb] = half_swap_max(mt[rb]);                      \
    }                                                                                                            \
    cur = nxt;                                                                                                   \
    nxt = nn;                                                                                                    \
  }

  for (int it = 0; it < n_tiles; it += 2) {
    DBSA_TILE_STEP(0, s_a, s_b)
    if (it + 1 >= n_tiles) break;
    ++it;
    DBSA_TILE_STEP(1, s_b, s_a)
    --it;
  }
#undef DBSA_TILE_STEP

  // ---- epilogue ----
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const float l_tot = half_swap_sum(l_run[rb]);
    if (!row_valid[rb]) continue;
    const float inv = 1.f / l_tot;
    __bf16* op = static_cast<__bf16*>(const_cast<void*>(p.o.ptr)) +
                 static_cast<int64_t>(row_tok[rb]) * p.o.stride_tok +
                 static_cast<int64_t>(head[rb]) * p.o.stride_head + 4 * half;
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
        *reinterpret_cast<bf16x4*>(op + 32 * ob + 8 * g) = w.v;
      }
    if (p.lse && half == 0)
      p.lse[static_cast<int64_t>(head[rb]) * p.lse_stride + row_tok[rb]] =
          (m_run[rb] + __log2f(l_tot)) * 0.69314718055994531f;
  }
}

template <int NW, int RB, bool SELF>
hipError_t launch_cfg(const AttnParams& p, hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_prefill_kernel<NW, RB, SELF>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  dim3 grid(p.n_q_heads / p.heads_per_block, p.n_qtiles), block(NW * 64);
  attn_prefill_kernel<NW, RB, SELF><<<grid, block, kLdsBytes, stream>>>(p);
  return hipGetLastError();
}

}  // namespace

// One workgroup takes heads_per_block * (block_m / 32) row blocks of 32 rows, one per wave.
hipError_t launch_prefill_pipelined(const AttnParams& p, hipStream_t stream) {
  if (p.n_qtiles == 0) return hipSuccess;
  const int row_blocks = p.heads_per_block * (p.block_m / 32);
  switch (row_blocks) {
    case 1: return p.query_stage ? launch_cfg<1, 1, true>(p, stream) : launch_cfg<1, 1, false>(p, stream);
    case 2: return p.query_stage ? launch_cfg<2, 1, true>(p, stream) : launch_cfg<2, 1, false>(p, stream);
    case 4: return p.query_stage ? launch_cfg<4, 1, true>(p, stream) : launch_cfg<4, 1, false>(p, stream);
    case 8: return p.query_stage ? launch_cfg<8, 1, true>(p, stream) : launch_cfg<8, 1, false>(p, stream);
    default: return hipErrorInvalidValue;
  }
}
