// Plain fp32-arithmetic attention kernels that walk the same tile lists as the MFMA
// kernels: one wavefront per (row, query head), one lane per key for the scores,
// one lane per output channel for the weighted sum.  They serve the DBSA_F32 dtype
// (fp32 storage, Sec. 2.1 / 2.2 semantics as documented in dbsa.h) and are not tuned.
// With a rotary table they also re-position (Sec. 2.2) for every shape the tuned kernels do not
// serve: the row of Q is rotated at list_shift[e] + (its index inside the Q tile) before it meets
// the keys of list entry e (decode: dec_shift[e] + self_len - 1, own cache: self_len - 1), anew
// wherever that id changes along the list.
#include "kernels.hpp"

namespace {

constexpr int kWave = 64;

__device__ inline float load_elem(const float* p) { return *p; }
__device__ inline float load_elem(const uint16_t* p) { return __uint_as_float(static_cast<uint32_t>(*p) << 16); }
__device__ inline void store_elem(float* p, float x) { *p = x; }
__device__ inline void store_elem(uint16_t* p, float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest even
  *p = static_cast<uint16_t>(u >> 16);
}

__device__ inline float wave_max(float x) {
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, kWave));
  return x;
}
__device__ inline float wave_sum(float x) {
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, kWave);
  return x;
}

// Running softmax state of one row, spread over a wavefront: lane owns output
// channels lane, lane+64, ...
template <int D>
struct RowState {
  float m = -INFINITY, l = 0.f;
  float acc[D / kWave] = {};
};

// Fold `count` keys starting at token `tok0` of (kbase, vbase) into the state.
// `limit`: keys with token index > limit are masked (pass INT_MAX for no mask).
template <typename T, int D>
__device__ void fold_keys(RowState<D>& st, const float* qs, const T* kbase, const T* vbase, int64_t stride_tok,
                          int tok0, int count, int limit, float scale) {
  const int lane = threadIdx.x % kWave;
  for (int c0 = 0; c0 < count; c0 += kWave) {
    const int n = min(kWave, count - c0);
    const int tok = tok0 + c0 + lane;
    const bool valid = lane < n && tok <= limit;
    float s = -INFINITY;
    if (valid) {
      const T* kr = kbase + static_cast<int64_t>(tok) * stride_tok;
      float dot = 0.f;
      for (int d = 0; d < D; ++d) dot = fmaf(qs[d], load_elem(kr + d), dot);
      s = dot * scale;
    }
    const float m_new = fmaxf(st.m, wave_max(s));
    if (m_new == -INFINITY) continue;  // nothing visible yet
    const float alpha = __expf(st.m - m_new);
    const float p = valid ? __expf(s - m_new) : 0.f;
    st.l = st.l * alpha + wave_sum(p);
    st.m = m_new;
#pragma unroll
    for (int i = 0; i < D / kWave; ++i) st.acc[i] *= alpha;
    for (int kk = 0; kk < n; ++kk) {
      const float pk = __shfl(p, kk, kWave);
      const T* vr = vbase + static_cast<int64_t>(tok0 + c0 + kk) * stride_tok;
#pragma unroll
      for (int i = 0; i < D / kWave; ++i) st.acc[i] = fmaf(pk, load_elem(vr + lane + i * kWave), st.acc[i]);
    }
  }
}

// qs = q0 rotated at id (channel i pairs with i + D/2; table = (cos, sin) per id and pair), one wavefront
template <int D>
__device__ void rotate_row(float* qs, const float* q0, const float* table, int id, int n_pos) {
  const int lane = threadIdx.x % kWave;
  const float* cs = table + static_cast<int64_t>(min(max(id, 0), n_pos - 1)) * D;
  __builtin_amdgcn_wave_barrier();  // the products that read the old qs are done
  for (int i = lane; i < D / 2; i += kWave) {
    const float c = cs[2 * i], sn = cs[2 * i + 1], a = q0[i], b = q0[i + D / 2];
    qs[i] = a * c - b * sn;
    qs[i + D / 2] = b * c + a * sn;
  }
  __builtin_amdgcn_wave_barrier();
}

template <typename T, int D, bool ROPE>
__global__ __launch_bounds__(256) void prefill_plain_kernel(AttnParams p) {
  __shared__ float qs_all[4][D];
  __shared__ float q0_all[ROPE ? 4 : 1][D];
  const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
  float* qs = qs_all[wave];
  float* q0 = ROPE ? q0_all[wave] : qs;
  const int tile = blockIdx.x, h = blockIdx.y;
  const int hk = h / (p.n_q_heads / p.n_kv_heads);
  const int q_start = p.qtile_tab[tile * 4 + 0], q_len = p.qtile_tab[tile * 4 + 1];
  const int64_t e0 = p.list_ptr[tile], e1 = p.list_ptr[tile + 1];
  const T* kp = static_cast<const T*>(p.k_pool.ptr) + hk * p.k_pool.stride_head;
  const T* vp = static_cast<const T*>(p.v_pool.ptr) + hk * p.v_pool.stride_head;
  const T* ks = static_cast<const T*>(p.k_self.ptr) + hk * p.k_self.stride_head;
  const T* vs = static_cast<const T*>(p.v_self.ptr) + hk * p.v_self.stride_head;
  for (int row = wave; row < q_len; row += 4) {
    const int tok = q_start + row;
    const T* qr = static_cast<const T*>(p.q.ptr) + static_cast<int64_t>(tok) * p.q.stride_tok + h * p.q.stride_head;
    for (int d = lane; d < D; d += kWave) q0[d] = load_elem(qr + d);
    __builtin_amdgcn_wave_barrier();
    RowState<D> st;
    int cur_id = INT_MIN;
    for (int64_t e = e0; e < e1; ++e) {
      const int kv_start = p.list_ent[2 * e], w1 = p.list_ent[2 * e + 1];
      const int kv_len = w1 & 0xFFFF, kind = w1 >> 16;
      if constexpr (ROPE) {
        const int id = p.list_shift[e] + row;
        if (id != cur_id) rotate_row<D>(qs, q0, p.rope_table, id, p.rope_n_pos);
        cur_id = id;
      }
      const bool self = kind & 2;
      const int limit = (kind & 1) ? tok : INT_MAX;
      fold_keys<T, D>(st, qs, self ? ks : kp, self ? vs : vp, self ? p.k_self.stride_tok : p.k_pool.stride_tok,
                      kv_start, kv_len, limit, p.scale);
    }
    T* orow = static_cast<T*>(const_cast<void*>(p.o.ptr)) + static_cast<int64_t>(tok) * p.o.stride_tok +
              h * p.o.stride_head;
    const float inv = 1.f / st.l;
#pragma unroll
    for (int i = 0; i < D / kWave; ++i) store_elem(orow + lane + i * kWave, st.acc[i] * inv);
    if (p.lse && lane == 0) p.lse[static_cast<int64_t>(h) * p.lse_stride + tok] = st.m + __logf(st.l);
    __builtin_amdgcn_wave_barrier();
  }
}

template <typename T, int D, bool ROPE>
__global__ __launch_bounds__(64) void decode_plain_kernel(AttnParams p) {
  __shared__ float qs[D];
  __shared__ float q0_sh[ROPE ? D : 1];
  float* q0 = ROPE ? q0_sh : qs;
  const int lane = threadIdx.x;
  const int u = blockIdx.x, h = blockIdx.y;
  const int hk = h / (p.n_q_heads / p.n_kv_heads);
  const T* qr = static_cast<const T*>(p.q.ptr) + static_cast<int64_t>(u) * p.q.stride_tok + h * p.q.stride_head;
  for (int d = lane; d < D; d += kWave) q0[d] = load_elem(qr + d);
  __builtin_amdgcn_wave_barrier();
  const int last = p.self_len[u] - 1;  // the new token's index inside the query
  int cur_id = INT_MIN;
  const T* kp = static_cast<const T*>(p.k_pool.ptr) + hk * p.k_pool.stride_head;
  const T* vp = static_cast<const T*>(p.v_pool.ptr) + hk * p.v_pool.stride_head;
  RowState<D> st;
  const int64_t e0 = p.split_ptr[static_cast<int64_t>(u) * (p.n_split + 1)];
  const int64_t e1 = p.split_ptr[static_cast<int64_t>(u) * (p.n_split + 1) + p.n_split];
  for (int64_t e = e0; e < e1; ++e) {
    const int kv_start = p.dec_ent[2 * e], kv_len = p.dec_ent[2 * e + 1] & 0xFFFF;
    if constexpr (ROPE) {
      const int id = p.dec_shift[e] + last;
      if (id != cur_id) rotate_row<D>(qs, q0, p.rope_table, id, p.rope_n_pos);
      cur_id = id;
    }
    fold_keys<T, D>(st, qs, kp, vp, p.k_pool.stride_tok, kv_start, kv_len, INT_MAX, p.scale);
  }
  if constexpr (ROPE) {
    if (last != cur_id) rotate_row<D>(qs, q0, p.rope_table, last, p.rope_n_pos);
  }
  const T* kc = static_cast<const T*>(p.k_self.ptr) + u * p.stride_query + hk * p.k_self.stride_head;
  const T* vc = static_cast<const T*>(p.v_self.ptr) + u * p.stride_query + hk * p.v_self.stride_head;
  fold_keys<T, D>(st, qs, kc, vc, p.k_self.stride_tok, 0, p.self_len[u], INT_MAX, p.scale);
  T* orow = static_cast<T*>(const_cast<void*>(p.o.ptr)) + static_cast<int64_t>(u) * p.o.stride_tok +
            h * p.o.stride_head;
  const float inv = 1.f / st.l;
#pragma unroll
  for (int i = 0; i < D / kWave; ++i) store_elem(orow + lane + i * kWave, st.acc[i] * inv);
}

}  // namespace

namespace {
template <typename T, int D>
void launch_prefill_as(const AttnParams& p, dim3 grid, dim3 block, hipStream_t stream) {
  if (p.rope_table)
    prefill_plain_kernel<T, D, true><<<grid, block, 0, stream>>>(p);
  else
    prefill_plain_kernel<T, D, false><<<grid, block, 0, stream>>>(p);
}
template <typename T, int D>
void launch_decode_as(const AttnParams& p, dim3 grid, dim3 block, hipStream_t stream) {
  if (p.rope_table)
    decode_plain_kernel<T, D, true><<<grid, block, 0, stream>>>(p);
  else
    decode_plain_kernel<T, D, false><<<grid, block, 0, stream>>>(p);
}
}  // namespace

hipError_t launch_prefill_plain(const AttnParams& p, int head_dim, bool bf16_storage, hipStream_t stream) {
  if (p.n_qtiles == 0) return hipSuccess;
  dim3 grid(p.n_qtiles, p.n_q_heads), block(256);
  if (head_dim == 64) {
    if (bf16_storage) launch_prefill_as<uint16_t, 64>(p, grid, block, stream);
    else launch_prefill_as<float, 64>(p, grid, block, stream);
  } else {
    if (bf16_storage) launch_prefill_as<uint16_t, 128>(p, grid, block, stream);
    else launch_prefill_as<float, 128>(p, grid, block, stream);
  }
  return hipGetLastError();
}

hipError_t launch_decode_plain(const AttnParams& p, int head_dim, bool bf16_storage, hipStream_t stream) {
  dim3 grid(p.n_queries, p.n_q_heads), block(64);
  if (head_dim == 64) {
    if (bf16_storage) launch_decode_as<uint16_t, 64>(p, grid, block, stream);
    else launch_decode_as<float, 64>(p, grid, block, stream);
  } else {
    if (bf16_storage) launch_decode_as<uint16_t, 128>(p, grid, block, stream);
    else launch_decode_as<float, 128>(p, grid, block, stream);
  }
  return hipGetLastError();
}
