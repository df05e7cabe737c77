// Software-pipelined bf16 MFMA attention for prefill-shaped calls (pre-encode, Sec. 2.1;
// query prefill, Sec. 2.2) at head_dim 128 on gfx950.  Same mathematics and register
// plan as attn_mfma.hip (transposed scores S^T = K Q^T, per-lane softmax statistics,
// O^T = V^T P^T); what differs is how the tiles move and how the work is ordered:
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
//   * the scores of tile j+1 are issued in the same straight-line region as the
//     exponentials of tile j, so the matrix pipe and the vector ALU overlap inside one
//     wave; the second product of tile j follows.
//   * a wave may own two 32-row blocks (64 rows): every K/V fragment read from LDS then
//     feeds two MFMAs, at one wave per SIMD with the full 512-register budget.
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
constexpr float kNegBig = -1.0e30f;
constexpr float kRescaleSlack = 8.f;

typedef __attribute__((address_space(3))) unsigned char lds_byte;

__device__ inline bf16x8 pack8(const floatx16& s, int first) {
  union {
    bf16x8 v;
    bf16x2 p[4];
  } u;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    u.p[i] = __builtin_convertvector(floatx2{s[first + 2 * i], s[first + 2 * i + 1]}, bf16x2);
  return u.v;
}

__device__ inline bf16x4 lds_read_tr(const lds_byte* p) {
  typedef __attribute__((address_space(3))) shortx4* tr_ptr;
  const shortx4 t = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(p));
  return __builtin_bit_cast(bf16x4, t);
}

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
__device__ inline void dma16(const void* gbase, unsigned byte_off, lds_byte* dst) {
  const unsigned m0v = static_cast<unsigned>(reinterpret_cast<uintptr_t>(dst));  // wave-uniform LDS address
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(m0v), "v"(byte_off), "s"(gbase)
               : "memory");
}

struct Tile {
  const __bf16* k;
  const __bf16* v;
  int64_t k_stride, v_stride;
  int kv_start, kv_len;
  bool causal;
};

// NW wavefronts per workgroup, RB 32-row blocks per wavefront.  Row block g = wave*RB + rb
// covers query head (blockIdx.y * heads_per_block + g / spb) and tokens
// q_start + (g % spb)*32 .. +31, spb = block_m / 32.
template <int NW, int RB>
__global__ __launch_bounds__(NW * 64, 2) void attn_prefill_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  constexpr int kBlocksPerWave = 16 / NW;  // 1-KiB load blocks of one operand per wave (NW <= 8 < 16)
  static_assert(NW == 1 || NW == 2 || NW == 4 || NW == 8, "wave count");
  lds_byte* lds = (lds_byte*)smem;

  const int tid = threadIdx.x, lane = tid % 64, l32 = lane % 32, half = lane / 32;
  const int wave = __builtin_amdgcn_readfirstlane(tid / 64);
  const int r = p.n_q_heads / p.n_kv_heads;

  // ---- rows of this wave, tiles of this workgroup ----
  const int tile = p.order[blockIdx.x];
  const int q_start = p.qtile_tab[tile * 4 + 0], q_len = p.qtile_tab[tile * 4 + 1];
  const int spb = p.block_m / 32;
  int head[RB], row_tok[RB], q_pos[RB], blk_q_hi[RB];
  bool row_valid[RB];
  bool wave_active = false;
  int wave_q_hi = 0;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int g = wave * RB + rb;
    const int sub = g % spb;
    head[rb] = blockIdx.y * p.heads_per_block + g / spb;
    const int row_local = sub * 32 + l32;
    row_valid[rb] = row_local < q_len;
    wave_active = wave_active || (sub * 32 < q_len);
    row_tok[rb] = q_start + min(row_local, q_len - 1);
    q_pos[rb] = q_start + row_local;
    blk_q_hi[rb] = q_start + sub * 32 + 31;
    wave_q_hi = max(wave_q_hi, blk_q_hi[rb]);
  }
  const int hk = (blockIdx.y * p.heads_per_block) / r;
  const int64_t e0 = p.list_ptr[tile];
  const int n_tiles = static_cast<int>(p.list_ptr[tile + 1] - e0);
  const int32_t* ent = p.list_ent + 2 * e0;

  const __bf16* kpool = static_cast<const __bf16*>(p.k_pool.ptr) + hk * p.k_pool.stride_head;
  const __bf16* vpool = static_cast<const __bf16*>(p.v_pool.ptr) + hk * p.v_pool.stride_head;
  const __bf16* kself = static_cast<const __bf16*>(p.k_self.ptr) + hk * p.k_self.stride_head;
  const __bf16* vself = static_cast<const __bf16*>(p.v_self.ptr) + hk * p.v_self.stride_head;

  auto tile_desc = [&](int it) {
    Tile t;
    const int w0 = ent[2 * it], w1 = ent[2 * it + 1];
    const int kind = w1 >> 16;
    const bool self = kind & 2;
    t.k = self ? kself : kpool;
    t.v = self ? vself : vpool;
    t.k_stride = self ? p.k_self.stride_tok : p.k_pool.stride_tok;
    t.v_stride = self ? p.v_self.stride_tok : p.v_pool.stride_tok;
    t.kv_start = w0;
    t.kv_len = w1 & 0xFFFF;
    t.causal = kind & 1;
    return t;
  };

  // ---- global -> LDS loads: this wave fills blocks wave*kBlocksPerWave .. of each operand ----
  // lane -> (row, slot) inside block b: row = 4*b + lane/16, slot = lane%16; the piece
  // fetched into that slot is column (slot ^ swizzle(row)).  4*b is a multiple of 4 and,
  // per wave, the blocks are consecutive, so the swizzles only depend on lane and j.
  auto issue_k = [&](const Tile& t, int stage) {
    const __bf16* base = t.k + static_cast<int64_t>(t.kv_start) * t.k_stride;  // uniform
#pragma unroll
    for (int j = 0; j < kBlocksPerWave; ++j) {
      const int b = wave * kBlocksPerWave + j;
      const int row_in = 4 * b + lane / 16;
      const int row = min(row_in, t.kv_len - 1);  // rows past the tail repeat the last key
      const int col = ((lane % 16) ^ (row_in % 16)) * 8;
      const unsigned off = static_cast<unsigned>(__mul24(row, static_cast<int>(t.k_stride)) + col) * 2u;
      dma16(base, off, lds + stage * kTileBytes + b * 1024);
    }
  };
  auto issue_v = [&](const Tile& t, int stage) {
    const __bf16* base = t.v + static_cast<int64_t>(t.kv_start) * t.v_stride;
#pragma unroll
    for (int j = 0; j < kBlocksPerWave; ++j) {
      const int b = wave * kBlocksPerWave + j;
      const int row_in = 4 * b + lane / 16;
      const int row = min(row_in, t.kv_len - 1);
      const int col = ((lane % 16) ^ (4 * (row_in % 4))) * 8;
      const unsigned off = static_cast<unsigned>(__mul24(row, static_cast<int>(t.v_stride)) + col) * 2u;
      dma16(base, off, lds + (2 + stage) * kTileBytes + b * 1024);
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

  // ---- Q^T fragments ----
  bf16x8 qf[RB][kD / 16];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const __bf16* qp = static_cast<const __bf16*>(p.q.ptr) + static_cast<int64_t>(row_tok[rb]) * p.q.stride_tok +
                       static_cast<int64_t>(head[rb]) * p.q.stride_head + 8 * half;
#pragma unroll
    for (int c = 0; c < kD / 16; ++c) qf[rb][c] = *reinterpret_cast<const bf16x8*>(qp + 16 * c);
  }

  floatx16 o[RB][kD / 32];
  float m_run[RB], l_run[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    m_run[rb] = kNegBig;
    l_run[rb] = 0.f;
#pragma unroll
    for (int ob = 0; ob < kD / 32; ++ob)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[rb][ob][i] = 0.f;
  }
  const float c2 = p.scale_log2e;

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
  // masks of a causal or short tile, applied to raw scores
  auto apply_mask = [&](floatx16 (&s)[RB][2], const Tile& t) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const int limit = t.causal ? (q_pos[rb] - t.kv_start) : kBN;  // visible iff key_local <= limit
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key_local = kb * 32 + 8 * (i / 4) + 4 * half + (i % 4);
          const bool vis = key_local < t.kv_len && key_local <= limit;
          s[rb][kb][i] = vis ? s[rb][kb][i] : -INFINITY;
        }
    }
  };

  // ---- prologue: K(0), V(0), K(1) in flight; scores and row maxima of tile 0 ----
  Tile cur{}, nxt{};
  floatx16 s_a[RB][2], s_b[RB][2];  // scores of the tile being consumed / of the next tile, swapping roles
  float mx_cur[RB];                 // scaled row maxima of the tile being consumed
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) mx_cur[rb] = -INFINITY;
  if (n_tiles > 0) {
    cur = tile_desc(0);
    issue_k(cur, 0);
    issue_v(cur, 0);
    if (n_tiles > 1) {
      nxt = tile_desc(1);
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
    if (cur.causal || cur.kv_len < kBN) apply_mask(s_a, cur);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float m = s_a[rb][0][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) m = fmaxf(m, s_a[rb][kb][i]);
      mx_cur[rb] = half_swap_max(m) * c2;
    }
  }

  // One tile step.  On entry s_cur / mx_cur hold the (masked) raw scores and scaled row
  // maxima of tile `it`; K(it+1) -> K stage 1-STAGE and V(it) -> V stage STAGE have been
  // issued.  The step issues the next loads, turns s_cur into probabilities while the
  // matrix pipe produces s_nxt, and accumulates O while the row maxima of s_nxt are
  // taken.  The last tile computes an s_nxt nobody uses (stale but finite-or-ignored LDS
  // contents) so that every tile runs the same straight-line code.
#define DBSA_TILE_STEP(STAGE, s_cur, s_nxt)                                                                      \
  {                                                                                                              \
    __builtin_amdgcn_s_waitcnt(0);                                                                               \
    __syncthreads();                                                                                             \
    Tile nn{};                                                                                                   \
    if (it + 2 < n_tiles) {                                                                                      \
      nn = tile_desc(it + 2);                                                                                    \
      issue_k(nn, STAGE);                                                                                        \
    }                                                                                                            \
    const bool has_next = it + 1 < n_tiles;                                                                      \
    if (has_next) issue_v(nxt, 1 - STAGE);                                                                       \
    /* The running max may lag the true max by kRescaleSlack (weights then reach 2^slack at most, */           \
    /* harmless in fp32/bf16): accumulators are rescaled only when some row of the wave outgrows it. */         \
    {                                                                                                            \
      bool grow = false;                                                                                         \
      _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) grow = grow || (mx_cur[rb] > m_run[rb] + kRescaleSlack); \
      if (__builtin_amdgcn_ballot_w64(grow) != 0) {                                                              \
        _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) {                                                      \
          const float m_new = fmaxf(m_run[rb], mx_cur[rb]);                                                      \
          const float alpha = __builtin_amdgcn_exp2f(m_run[rb] - m_new);                                         \
          m_run[rb] = m_new;                                                                                     \
          l_run[rb] *= alpha;                                                                                    \
          _Pragma("unroll") for (int ob = 0; ob < kD / 32; ++ob) o[rb][ob] *= alpha;                             \
        }                                                                                                        \
      }                                                                                                          \
    }                                                                                                            \
    /* -- scores of the next tile (matrix pipe) || probabilities of this tile (vector ALU) -- */                \
    bf16x2 pk[RB][2][8];                                                                                         \
    float psum[RB];                                                                                              \
    _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) {                                                          \
      psum[rb] = 0.f;                                                                                            \
      _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) _Pragma("unroll") for (int i = 0; i < 16; ++i)            \
          s_nxt[rb][kb][i] = 0.f;                                                                                \
    }                                                                                                            \
    {                                                                                                            \
      bf16x8 kf[3];                                                                                              \
      kf[0] = ld_k(1 - STAGE, 0);                                                                                \
      kf[1] = ld_k(1 - STAGE, 1);                                                                                \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
      _Pragma("unroll") for (int t = 0; t < 16; ++t) {                                                           \
        if (t + 2 < 16) kf[(t + 2) % 3] = ld_k(1 - STAGE, t + 2);                                                \
        _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) s_nxt[rb][t / 8] =                                     \
            __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t % 3], qf[rb][t % 8], s_nxt[rb][t / 8], 0, 0, 0);        \
        _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) {                                                      \
          const int kb = t / 8, i = 2 * (t % 8);                                                                 \
          const float p0 = __builtin_amdgcn_exp2f(fmaf(s_cur[rb][kb][i], c2, -m_run[rb]));                       \
          const float p1 = __builtin_amdgcn_exp2f(fmaf(s_cur[rb][kb][i + 1], c2, -m_run[rb]));                   \
          psum[rb] += p0 + p1;                                                                                   \
          pk[rb][kb][t % 8] = __builtin_convertvector(floatx2{p0, p1}, bf16x2);                                  \
        }                                                                                                        \
        __builtin_amdgcn_sched_barrier(0);                                                                       \
      }                                                                                                          \
    }                                                                                                            \
    _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) l_run[rb] += psum[rb];                                     \
    if (has_next && (nxt.causal || nxt.kv_len < kBN)) apply_mask(s_nxt, nxt);                                    \
    /* -- O^T += V^T P^T (matrix pipe) || row maxima of the next tile (vector ALU) -- */                        \
    {                                                                                                            \
      float mt[RB];                                                                                              \
      _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) mt[rb] = s_nxt[rb][0][0];                                \
      bf16x8 vf[3];                                                                                              \
      vf[0] = ld_v(STAGE, 0);                                                                                    \
      vf[1] = ld_v(STAGE, 1);                                                                                    \
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
        }                                                                                                        \
        __builtin_amdgcn_sched_barrier(0);                                                                       \
      }                                                                                                          \
      _Pragma("unroll") for (int rb = 0; rb < RB; ++rb) mx_cur[rb] = half_swap_max(mt[rb]) * c2;                 \
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
  (void)wave_active;
  (void)wave_q_hi;

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

template <int NW, int RB>
hipError_t launch_cfg(const AttnParams& p, hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_prefill_kernel<NW, RB>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  dim3 grid(p.n_qtiles, p.n_q_heads / p.heads_per_block), block(NW * 64);
  attn_prefill_kernel<NW, RB><<<grid, block, kLdsBytes, stream>>>(p);
  return hipGetLastError();
}

}  // namespace

// One workgroup takes heads_per_block * (block_m / 32) row blocks of 32 rows, one per wave.
// (Measured on MI355X: one wave per SIMD issues MFMA and VALU work at only half the peak
// rate, so two row blocks per wave at one wave per SIMD is not used.)
hipError_t launch_prefill_pipelined(const AttnParams& p, hipStream_t stream) {
  if (p.n_qtiles == 0) return hipSuccess;
  const int row_blocks = p.heads_per_block * (p.block_m / 32);
  switch (row_blocks) {
    case 1: return launch_cfg<1, 1>(p, stream);
    case 2: return launch_cfg<2, 1>(p, stream);
    case 4: return launch_cfg<4, 1>(p, stream);
    case 8: return launch_cfg<8, 1>(p, stream);
    default: return hipErrorInvalidValue;
  }
}
