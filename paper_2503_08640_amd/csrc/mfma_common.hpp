// Device helpers shared by the bf16 MFMA kernels (attn_prefill.hip, attn_prefill64.hip,
// attn_decode.hip, attn_mfma.hip): vector typedefs, LDS transpose reads, half-wave exchanges,
// asynchronous global -> LDS loads and explicit waits, the query-row loader of the 32-column
// kernels.  Nothing here is specific to one kernel.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>
#include <utility>

namespace dbsa_mfma {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef short shortx4 __attribute__((ext_vector_type(4)));

typedef __attribute__((address_space(3))) unsigned char lds_byte;
typedef const __attribute__((address_space(4))) int32_t* const_words;  // read-only lists: scalar loads

#define DBSA_INLINE __attribute__((always_inline))

// calls f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): loops whose index must
// stay a compile-time constant (register arrays, immediate LDS offsets)
template <typename F, int... I>
__device__ DBSA_INLINE void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ DBSA_INLINE void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// ds_read_b64_tr_b16: within a group of 16 lanes, lane i supplies the address of one key's four
// channels and receives four keys of one channel (the transposed operand of the PV product).
__device__ inline bf16x4 lds_read_tr(const lds_byte* p) {
  typedef __attribute__((address_space(3))) shortx4* tr_ptr;
  const shortx4 t = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(p));
  return __builtin_bit_cast(bf16x4, t);
}

// the same through a generic pointer into LDS
__device__ inline bf16x4 lds_read_tr(const __bf16* p) {
  typedef __attribute__((address_space(3))) shortx4* tr_ptr;
  const shortx4 t = __builtin_amdgcn_ds_read_tr16_b64_v4i16((tr_ptr)(p));
  return __builtin_bit_cast(bf16x4, t);
}

// Combine a value held by lanes l and l^32 (the two half-waves hold the two key halves of
// the same score column).
__device__ inline float half_swap_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float half_swap_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// A wave-uniform 64-bit value, in scalar registers as far as the compiler is concerned.
// (readfirstlane returns a signed int: widen through unsigned, or the low word would be sign-extended)
__device__ inline uint64_t uniform64(uint64_t x) {
  const unsigned hi = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(x >> 32)));
  const unsigned lo = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(x & 0xFFFFFFFFu)));
  return (static_cast<uint64_t>(hi) << 32) | static_cast<uint64_t>(lo);
}

// 16 bytes per lane from global memory straight into LDS: lane l's piece lands at LDS byte
// address lds_addr + 16*l.  Issued through inline assembly so that the transfer stays
// asynchronous: the kernels wait for it explicitly (vmcnt) where the data is needed, instead
// of before the next LDS read of any kind.  gbase and lds_addr are wave-uniform and must reach
// the instruction in scalar registers (uniform64, readfirstlane); m0 carries the LDS address.
// m0 cannot be named as a clobber (it is a reserved register: the compiler warns and ignores the
// entry), so the kernels that include this header use nothing for which the COMPILER keeps a value
// of its own in m0 across statements: no LDS-DMA or LDS-direct builtins, no sendmsg, no indirect
// register indexing.  The assembly re-loads m0 before every transfer and relies on no earlier value.
__device__ inline void dma16(uint64_t gbase, unsigned byte_off, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(byte_off), "s"(gbase)
               : "memory");
}

// The same for callers that hold a global pointer and an LDS pointer whose uniformity the compiler
// cannot see: both are made scalar here.
__device__ inline void dma16(const void* gbase, unsigned byte_off, lds_byte* dst) {
  const unsigned m0v = static_cast<unsigned>(
      __builtin_amdgcn_readfirstlane(static_cast<int>(reinterpret_cast<uintptr_t>(dst) & 0xFFFFFFFFu)));
  dma16(uniform64(reinterpret_cast<uint64_t>(gbase)), byte_off, m0v);
}

// Wait until at most N vector-memory operations of this wave are outstanding (they complete
// in issue order).  The memory clobber keeps LDS accesses of the awaited data below the wait.
template <int N>
__device__ inline void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// The 8 B-operand fragments of one score column for head_dim 128: the query row (qp points at this
// lane's first channel, 8 * half), pre-multiplied by c2 = scale * log2 e and rounded to bf16 again.
// ROPE: the row is stored un-rotated and is rotated here with the table row `rot` (16 floats = cos,
// sin of 8 channel pairs per (chunk, half)); channel d < 64 of chunk c pairs with channel d + 64 of
// chunk c + 4, both held by this lane.
template <bool ROPE>
__device__ DBSA_INLINE void load_query_fragments(const __bf16* qp, const float* rot, float c2, bf16x8 (&qf)[8]) {
  constexpr int kQD = 128;
  if (ROPE) {
#pragma unroll
    for (int c = 0; c < kQD / 32; ++c) {
      const bf16x8 lo = *reinterpret_cast<const bf16x8*>(qp + 16 * c);
      const bf16x8 hi = *reinterpret_cast<const bf16x8*>(qp + 16 * (c + kQD / 32));
      floatx4 cs[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) cs[j] = *reinterpret_cast<const floatx4*>(rot + 32 * c + 4 * j);
      union {
        bf16x8 v;
        bf16x2 p2[4];
      } a, b;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float x0 = static_cast<float>(lo[2 * e]), y0 = static_cast<float>(hi[2 * e]);
        const float x1 = static_cast<float>(lo[2 * e + 1]), y1 = static_cast<float>(hi[2 * e + 1]);
        const float c0 = cs[e][0] * c2, s0 = cs[e][1] * c2, c1 = cs[e][2] * c2, s1 = cs[e][3] * c2;
        a.p2[e] = __builtin_convertvector(floatx2{x0 * c0 - y0 * s0, x1 * c1 - y1 * s1}, bf16x2);
        b.p2[e] = __builtin_convertvector(floatx2{y0 * c0 + x0 * s0, y1 * c1 + x1 * s1}, bf16x2);
      }
      qf[c] = a.v;
      qf[c + kQD / 32] = b.v;
    }
  } else {
#pragma unroll
    for (int c = 0; c < kQD / 16; ++c) {
      const bf16x8 raw = *reinterpret_cast<const bf16x8*>(qp + 16 * c);
      union {
        bf16x8 v;
        bf16x2 p2[4];
      } sc;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        sc.p2[e] = __builtin_convertvector(
            floatx2{static_cast<float>(raw[2 * e]) * c2, static_cast<float>(raw[2 * e + 1]) * c2}, bf16x2);
      qf[c] = sc.v;
    }
  }
}

}  // namespace dbsa_mfma
