// Device helpers shared by the bf16 MFMA kernels (attn_prefill.hip, attn_prefill64.hip,
// attn_decode.hip, attn_mfma.hip): vector typedefs, LDS transpose reads, half-wave exchanges,
// asynchronous global -> LDS loads and explicit waits.  Nothing here is specific to one kernel.
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
__device__ inline void dma16(uint64_t gbase, unsigned byte_off, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(byte_off), "s"(gbase)
               : "memory");
}

// Wait until at most N vector-memory operations of this wave are outstanding (they complete
// in issue order).  The memory clobber keeps LDS accesses of the awaited data below the wait.
template <int N>
__device__ inline void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

}  // namespace dbsa_mfma
