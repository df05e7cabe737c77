// Rotary position tables and the encoding-time rotation of keys (Sec. 2.1: the pool is encoded
// with sequential position ids; Sec. 2.2: new in-order ids at query time).  Convention of the
// Llama models the paper runs: channel i pairs with channel i + D/2, angle = id * inv_freq[i].
#include <cstdint>

#include "kernels.hpp"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct FreqArg {
  double f[64];
};

// table[n][i] = (cos, sin)(n * inv_freq[i]) rounded to fp32 from an fp64 evaluation: the angle
// reaches ~1e5 rad at the pool sizes in question, where an fp32 product would already be off
// by several 1e-3 rad.
__global__ void rope_table_kernel(FreqArg fr, int half_dim, int n_pos, float* table) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= static_cast<int64_t>(n_pos) * half_dim) return;
  const int n = static_cast<int>(idx / half_dim), i = static_cast<int>(idx % half_dim);
  const double ang = static_cast<double>(n) * fr.f[i];
  double s, c;
  sincos(ang, &s, &c);
  table[2 * idx] = static_cast<float>(c);
  table[2 * idx + 1] = static_cast<float>(s);
}

// one thread rotates 8 channel pairs (i .. i+7, partners at + D/2) of one (token, head)
template <typename T>
__global__ void rope_apply_kernel(const T* x, int64_t x_tok, int64_t x_head, T* out, int64_t o_tok, int64_t o_head,
                                  int n_tokens, int n_heads, int half_dim, const int32_t* positions, int first_id,
                                  const float* table, int n_pos) {
  const int per_row = half_dim / 8;
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (idx >= static_cast<int64_t>(n_tokens) * n_heads * per_row) return;
  const int part = static_cast<int>(idx % per_row);
  const int head = static_cast<int>((idx / per_row) % n_heads);
  const int tok = static_cast<int>(idx / (static_cast<int64_t>(per_row) * n_heads));
  int id = positions ? positions[tok] : first_id + tok;
  id = min(max(id, 0), n_pos - 1);
  const float* cs = table + (static_cast<int64_t>(id) * half_dim + 8 * part) * 2;
  const T* xp = x + tok * x_tok + head * x_head + 8 * part;
  T* op = out + tok * o_tok + head * o_head + 8 * part;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float a = static_cast<float>(xp[e]), b = static_cast<float>(xp[e + half_dim]);
    const float c = cs[2 * e], s = cs[2 * e + 1];
    op[e] = static_cast<T>(a * c - b * s);
    op[e + half_dim] = static_cast<T>(b * c + a * s);
  }
}

}  // namespace

hipError_t launch_rope_table(const double* inv_freq, int head_dim, int n_pos, float* table, hipStream_t stream) {
  FreqArg fr{};
  for (int i = 0; i < head_dim / 2; ++i) fr.f[i] = inv_freq[i];
  const int64_t n = static_cast<int64_t>(n_pos) * (head_dim / 2);
  if (n == 0) return hipSuccess;
  rope_table_kernel<<<static_cast<unsigned>((n + 255) / 256), 256, 0, stream>>>(fr, head_dim / 2, n_pos, table);
  return hipGetLastError();
}

hipError_t launch_rope_apply(const TensorView& x, const TensorView& out, int n_tokens, int n_heads, int head_dim,
                             bool bf16, const int32_t* positions, int first_id, const float* table, int n_pos,
                             hipStream_t stream) {
  const int64_t n = static_cast<int64_t>(n_tokens) * n_heads * (head_dim / 16);
  if (n == 0) return hipSuccess;
  const unsigned grid = static_cast<unsigned>((n + 255) / 256);
  if (bf16)
    rope_apply_kernel<__bf16><<<grid, 256, 0, stream>>>(
        static_cast<const __bf16*>(x.ptr), x.stride_tok, x.stride_head,
        static_cast<__bf16*>(const_cast<void*>(out.ptr)), out.stride_tok, out.stride_head, n_tokens, n_heads,
        head_dim / 2, positions, first_id, table, n_pos);
  else
    rope_apply_kernel<float><<<grid, 256, 0, stream>>>(
        static_cast<const float*>(x.ptr), x.stride_tok, x.stride_head, static_cast<float*>(const_cast<void*>(out.ptr)),
        out.stride_tok, out.stride_head, n_tokens, n_heads, head_dim / 2, positions, first_id, table, n_pos);
  return hipGetLastError();
}
