// bf16 MFMA flash-style attention kernels for gfx950 that walk only the KV tiles a
// layout lists (Sec. 2.1: masked blocks are skipped; Sec. 2.2: the selected groups'
// KV is read in place).
//
// Register plan per wavefront (64 lanes, v_mfma_f32_32x32x16_bf16):
//   * the wave owns 32 rows (query tokens of one head; at decode the r heads of one
//     KV head) and keeps Q^T as the B operand: lane (n = lane%32, half = lane/32)
//     holds channels 16c + 8*half .. +7 of row n for every 16-channel chunk c.
//   * scores are produced TRANSPOSED, S^T = K Q^T, 32 keys x 32 rows per MFMA
//     accumulator: lane holds row n and the 16 keys 8*(reg/4) + 4*half + reg%4.
//     A row's softmax statistics are therefore per lane (plus one exchange between
//     the two half-waves), and the probabilities are already laid out as the B
//     operand of the second product without any cross-lane movement.
//   * the output is accumulated transposed too, O^T = V^T P^T, so that rescaling by
//     the running-max correction is a per-lane scalar multiply.
// K and V tiles sit in LDS row-major with padded rows.  The second product needs, per
// lane, 4 consecutive keys of one channel: that transposed fragment comes from the
// gfx950 LDS transpose read (ds_read_b64_tr_b16), in which lane i of a 16-lane group
// supplies the address of key k0 + i/4, channels c0 + 4*(i%4).. and receives keys
// k0..k0+3 of channel c0 + i.
#include "kernels.hpp"
#include "mfma_common.hpp"

namespace {

using namespace dbsa_mfma;

typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

constexpr int kBN = 64;            // keys per KV tile
constexpr float kNegBig = -1.0e30f;  // "no key seen yet" running max (finite on purpose)

template <int D>
struct Lds {
  static constexpr int kKStride = D + 8;   // elements per K row: 16 B of padding (rows shift by 4 banks)
  static constexpr int kVStride = D + 32;  // elements per V row: 64 B of padding (rows shift by 16 banks):
                                           // measured conflict-free for the transpose reads
  static constexpr int kBytes = (kBN * kKStride + kBN * kVStride) * 2;
};

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

constexpr float kRescaleSlack = 8.f;  // log2 units the running max may lag before accumulators are rescaled

struct TileDesc {
  const __bf16* k;  // row 0 of the tile for this KV head
  const __bf16* v;
  int64_t k_stride, v_stride;  // elements between tokens
  int kv_start, kv_len;
  bool causal;
};

template <int D, int NW, bool DECODE>
__global__ __launch_bounds__(NW * 64) void attn_mfma_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using L = Lds<D>;
  constexpr int NT = NW * 64;
  constexpr int kPiecesPerRow = D / 8;            // 16-byte pieces per K/V row
  constexpr int PPT = kBN * kPiecesPerRow / NT;   // pieces each thread moves per tile
  static_assert(PPT >= 1 && PPT * NT == kBN * kPiecesPerRow, "tile must split evenly over the workgroup");
  __bf16* lds_k = reinterpret_cast<__bf16*>(smem);
  __bf16* lds_v = lds_k + kBN * L::kKStride;

  const int tid = threadIdx.x, wave = tid / 64, lane = tid % 64, l32 = lane % 32, half = lane / 32;
  const int r = p.n_q_heads / p.n_kv_heads;

  // ---- which rows does this wave own, and which tiles does the workgroup walk ----
  int head, hk, row_tok, q_pos;  // q_pos: token index used by the causal compare
  int wave_q_hi = 0;             // largest q_pos over the wave's rows
  bool row_valid, wave_active;
  int64_t e0, e1;
  int n_self_tiles = 0, self_len = 0, u = 0, split = 0;
  const int32_t* ent;
  if constexpr (!DECODE) {
    const int tile = p.order[blockIdx.x];
    const int q_start = p.qtile_tab[tile * 4 + 0], q_len = p.qtile_tab[tile * 4 + 1];
    const int spb = p.block_m / 32;
    const int sub = wave % spb;
    head = blockIdx.y * p.heads_per_block + wave / spb;
    hk = head / r;
    const int row_local = sub * 32 + l32;
    row_valid = row_local < q_len;
    wave_active = sub * 32 < q_len;
    row_tok = q_start + min(row_local, q_len - 1);
    q_pos = q_start + row_local;
    wave_q_hi = q_start + sub * 32 + 31;
    e0 = p.list_ptr[tile];
    e1 = p.list_ptr[tile + 1];
    ent = p.list_ent;
  } else {
    split = blockIdx.x;
    hk = blockIdx.y;
    u = blockIdx.z;
    head = hk * r + min(l32, r - 1);
    row_valid = l32 < r;
    wave_active = true;
    row_tok = u;
    q_pos = 0;
    e0 = p.split_ptr[static_cast<int64_t>(u) * (p.n_split + 1) + split];
    e1 = p.split_ptr[static_cast<int64_t>(u) * (p.n_split + 1) + split + 1];
    ent = p.dec_ent;
    if (split == p.n_split - 1) {
      self_len = p.self_len[u];
      n_self_tiles = (self_len + kBN - 1) / kBN;
    }
  }
  const int n_tiles = static_cast<int>(e1 - e0) + n_self_tiles;

  const __bf16* kpool = static_cast<const __bf16*>(p.k_pool.ptr) + hk * p.k_pool.stride_head;
  const __bf16* vpool = static_cast<const __bf16*>(p.v_pool.ptr) + hk * p.v_pool.stride_head;
  const __bf16* kself = static_cast<const __bf16*>(p.k_self.ptr) + hk * p.k_self.stride_head +
                        (DECODE ? u * p.stride_query : 0);
  const __bf16* vself = static_cast<const __bf16*>(p.v_self.ptr) + hk * p.v_self.stride_head +
                        (DECODE ? u * p.stride_query : 0);

  auto tile_desc = [&](int it) {
    TileDesc t;
    const int n_listed = static_cast<int>(e1 - e0);
    if (it < n_listed) {
      const int w0 = ent[2 * (e0 + it)], w1 = ent[2 * (e0 + it) + 1];
      const int kind = w1 >> 16;
      const bool self = kind & 2;
      t.k = self ? kself : kpool;
      t.v = self ? vself : vpool;
      t.k_stride = self ? p.k_self.stride_tok : p.k_pool.stride_tok;
      t.v_stride = self ? p.v_self.stride_tok : p.v_pool.stride_tok;
      t.kv_start = w0;
      t.kv_len = w1 & 0xFFFF;
      t.causal = kind & 1;
    } else {  // decode: the query's own cached keys, all visible
      const int s0 = (it - n_listed) * kBN;
      t.k = kself;
      t.v = vself;
      t.k_stride = p.k_self.stride_tok;
      t.v_stride = p.v_self.stride_tok;
      t.kv_start = s0;
      t.kv_len = min(kBN, self_len - s0);
      t.causal = false;
    }
    return t;
  };

  // ---- Q^T fragments ----
  bf16x8 qf[D / 16];
  {
    const __bf16* qp = static_cast<const __bf16*>(p.q.ptr) + static_cast<int64_t>(row_tok) * p.q.stride_tok +
                       static_cast<int64_t>(head) * p.q.stride_head + 8 * half;
#pragma unroll
    for (int c = 0; c < D / 16; ++c) qf[c] = *reinterpret_cast<const bf16x8*>(qp + 16 * c);
  }

  floatx16 o[D / 32];
#pragma unroll
  for (int ob = 0; ob < D / 32; ++ob)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[ob][i] = 0.f;
  float m_run = kNegBig, l_run = 0.f;  // running max (log2 domain, scaled) and this lane's share of the sum
  const float c2 = p.scale_log2e;

  // ---- global -> register prefetch of one K/V tile, then registers -> LDS ----
  uintx4 kreg[PPT], vreg[PPT];
#define DBSA_PREFETCH(t)                                                                                       \
  _Pragma("unroll") for (int j = 0; j < PPT; ++j) {                                                            \
    const int piece = tid + j * NT;                                                                            \
    const int row = min(piece / kPiecesPerRow, (t).kv_len - 1); /* rows past the tail repeat the last key */   \
    const int col = (piece % kPiecesPerRow) * 8;                                                               \
    kreg[j] = *reinterpret_cast<const uintx4*>((t).k + static_cast<int64_t>((t).kv_start + row) * (t).k_stride + col); \
    vreg[j] = *reinterpret_cast<const uintx4*>((t).v + static_cast<int64_t>((t).kv_start + row) * (t).v_stride + col); \
  }
#define DBSA_STAGE()                                                                   \
  _Pragma("unroll") for (int j = 0; j < PPT; ++j) {                                    \
    const int piece = tid + j * NT;                                                    \
    const int row = piece / kPiecesPerRow, col = (piece % kPiecesPerRow) * 8;          \
    *reinterpret_cast<uintx4*>(lds_k + row * L::kKStride + col) = kreg[j];              \
    *reinterpret_cast<uintx4*>(lds_v + row * L::kVStride + col) = vreg[j];              \
  }

  // this lane's address inside a V tile for the transpose reads: key 4*half + (i/4),
  // channel 16*(l32/16) + 4*(i%4), i = lane%16
  const __bf16* v_lane = lds_v + (4 * half + (lane % 16) / 4) * L::kVStride + 16 * (l32 / 16) + 4 * (lane % 4);

  TileDesc cur{}, nxt{};
  if (n_tiles > 0) {
    nxt = tile_desc(0);
    DBSA_PREFETCH(nxt)
  }
  for (int it = 0; it < n_tiles; ++it) {
    cur = nxt;
    __syncthreads();  // every wave has finished reading the previous tile
    DBSA_STAGE()
    __syncthreads();
    if (it + 1 < n_tiles) {
      nxt = tile_desc(it + 1);
      DBSA_PREFETCH(nxt)
    }
    if (!wave_active) continue;

    // 32-key blocks of this tile that hold a key visible to some row of the wave
    int nkb = (cur.kv_len + 31) / 32;
    if (cur.causal) nkb = max(0, min(nkb, (wave_q_hi - cur.kv_start) / 32 + 1));
    if (wave_q_hi < cur.kv_start && cur.causal) nkb = 0;
    if (nkb == 0) continue;

    // S^T = K Q^T
    floatx16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
      if (kb < nkb) {
        const __bf16* kp = lds_k + (kb * 32 + l32) * L::kKStride + 8 * half;
#pragma unroll
        for (int c = 0; c < D / 16; ++c) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(kp + 16 * c);
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[c], s[kb], 0, 0, 0);
        }
      }
    }
    if (cur.causal || cur.kv_len < kBN) {
      const int limit = cur.causal ? (q_pos - cur.kv_start) : kBN;  // visible iff key_local <= limit
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key_local = kb * 32 + 8 * (i / 4) + 4 * half + (i % 4);
          const bool vis = key_local < cur.kv_len && key_local <= limit;
          s[kb][i] = vis ? s[kb][i] : -INFINITY;
        }
    }
    // online softmax, one row per lane (two lanes per row: exchange across half-waves)
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
      if (kb < nkb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kb][i]);
      }
    mx = half_swap_max(mx) * c2;
    // The running max may lag the true max by kRescaleSlack (the weights then reach
    // 2^slack at most, harmless in fp32/bf16): accumulators are rescaled only when some
    // row of the wave outgrows it, which is rare once a few tiles have been seen.
    if (__builtin_amdgcn_ballot_w64(mx > m_run + kRescaleSlack) != 0) {
      const float m_new = fmaxf(m_run, mx);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int ob = 0; ob < D / 32; ++ob) o[ob] *= alpha;
    }
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
      if (kb < nkb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          s[kb][i] = __builtin_amdgcn_exp2f(fmaf(s[kb][i], c2, -m_run));
          psum += s[kb][i];
        }
      }
    l_run += psum;
    // O^T += V^T P^T
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
      if (kb < nkb) {
#pragma unroll
        for (int ch = 0; ch < 2; ++ch) {
          const bf16x8 pf = pack8(s[kb], 8 * ch);
#pragma unroll
          for (int ob = 0; ob < D / 32; ++ob) {
            const __bf16* vp = v_lane + (kb * 32 + 16 * ch) * L::kVStride + 32 * ob;
            const bf16x4 lo = lds_read_tr(vp);
            const bf16x4 hi = lds_read_tr(vp + 8 * L::kVStride);
            const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            o[ob] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf, o[ob], 0, 0, 0);
          }
        }
      }
  }

#undef DBSA_PREFETCH
#undef DBSA_STAGE

  // ---- epilogue ----
  const float l_tot = half_swap_sum(l_run);
  if (!row_valid) return;
  if constexpr (!DECODE) {
    const float inv = 1.f / l_tot;
    __bf16* op = static_cast<__bf16*>(const_cast<void*>(p.o.ptr)) + static_cast<int64_t>(row_tok) * p.o.stride_tok +
                 static_cast<int64_t>(head) * p.o.stride_head + 4 * half;
#pragma unroll
    for (int ob = 0; ob < D / 32; ++ob)
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
  } else {
    float* part = p.partial + ((static_cast<int64_t>(u) * p.n_split + split) * p.n_q_heads + head) * (D + kPartialPad);
#pragma unroll
    for (int ob = 0; ob < D / 32; ++ob)
#pragma unroll
      for (int i = 0; i < 16; ++i) part[32 * ob + 8 * (i / 4) + 4 * half + (i % 4)] = o[ob][i];
    if (half == 0) {
      part[D] = m_run;
      part[D + 1] = l_tot;
    }
  }
}

// Second decode pass: fold the per-split states of one (query, head) into the output,
//   m* = max_s m_s ; l* = sum_s l_s 2^(m_s - m*) ; o = sum_s acc_s 2^(m_s - m*) / l*
// (running maxima are kept in the log2 domain, hence base 2).
template <int D, bool OUT_BF16>
__global__ __launch_bounds__(D) void decode_merge_kernel(AttnParams p) {
  const int u = blockIdx.x / p.n_q_heads, head = blockIdx.x % p.n_q_heads, d = threadIdx.x;
  constexpr int kRow = D + kPartialPad;
  const int64_t slot_stride = static_cast<int64_t>(p.n_q_heads) * kRow;
  const float* part = p.partial + static_cast<int64_t>(u) * p.n_split * slot_stride + static_cast<int64_t>(head) * kRow;
  float m_star = kNegBig;
  for (int s = 0; s < p.n_split; ++s) m_star = fmaxf(m_star, part[s * slot_stride + D]);
  float l_star = 0.f, acc = 0.f;
  for (int s = 0; s < p.n_split; ++s) {
    const float w = __builtin_amdgcn_exp2f(part[s * slot_stride + D] - m_star);
    l_star = fmaf(part[s * slot_stride + D + 1], w, l_star);
    acc = fmaf(part[s * slot_stride + d], w, acc);
  }
  const float out = acc / l_star;
  void* obase = const_cast<void*>(p.o.ptr);
  const int64_t off = static_cast<int64_t>(u) * p.o.stride_tok + static_cast<int64_t>(head) * p.o.stride_head + d;
  if constexpr (OUT_BF16)
    static_cast<__bf16*>(obase)[off] = static_cast<__bf16>(out);
  else
    static_cast<float*>(obase)[off] = out;
}

template <int D, int NW>
hipError_t launch_prefill_nw(const AttnParams& p, hipStream_t stream) {
  dim3 grid(p.n_qtiles, p.n_q_heads / p.heads_per_block), block(NW * 64);
  attn_mfma_kernel<D, NW, false><<<grid, block, Lds<D>::kBytes, stream>>>(p);
  return hipGetLastError();
}

template <int D>
hipError_t launch_prefill_d(const AttnParams& p, hipStream_t stream) {
  const int nw = p.heads_per_block * (p.block_m / 32);
  switch (nw) {
    case 1: return launch_prefill_nw<D, 1>(p, stream);
    case 2: return launch_prefill_nw<D, 2>(p, stream);
    case 4: return launch_prefill_nw<D, 4>(p, stream);
    case 8: return launch_prefill_nw<D, 8>(p, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

hipError_t launch_prefill_mfma(const AttnParams& p, int head_dim, hipStream_t stream) {
  if (p.n_qtiles == 0) return hipSuccess;
  return head_dim == 64 ? launch_prefill_d<64>(p, stream) : launch_prefill_d<128>(p, stream);
}

hipError_t launch_decode_mfma(const AttnParams& p, int head_dim, hipStream_t stream) {
  dim3 grid(p.n_split, p.n_kv_heads, p.n_queries), block(64);
  if (head_dim == 64)
    attn_mfma_kernel<64, 1, true><<<grid, block, Lds<64>::kBytes, stream>>>(p);
  else
    attn_mfma_kernel<128, 1, true><<<grid, block, Lds<128>::kBytes, stream>>>(p);
  return hipGetLastError();
}

hipError_t launch_decode_merge(const AttnParams& p, int head_dim, bool out_bf16, hipStream_t stream) {
  dim3 grid(p.n_queries * p.n_q_heads), block(head_dim);
  if (head_dim == 64) {
    if (out_bf16) decode_merge_kernel<64, true><<<grid, block, 0, stream>>>(p);
    else decode_merge_kernel<64, false><<<grid, block, 0, stream>>>(p);
  } else {
    if (out_bf16) decode_merge_kernel<128, true><<<grid, block, 0, stream>>>(p);
    else decode_merge_kernel<128, false><<<grid, block, 0, stream>>>(p);
  }
  return hipGetLastError();
}
