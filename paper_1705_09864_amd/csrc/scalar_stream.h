// Scalar-operand streaming for the xor/popcount kernels.
//
// The operand that is the same for every lane of a wave (a filter row, a block of
// activation rows) never needs vector registers or vector loads: it is fetched with scalar
// loads into SGPRs and enters v_xor_b32 / v_and_b32 as the scalar source.  This header holds
// the pieces both the convolution and the GEMM kernels use for that.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bmx {

// Wave-uniform read-only data (filter rows, alpha) is read through the constant address
// space so that the loads are scalar (s_load into SGPRs) and never occupy vector lanes.
typedef const uint32_t __attribute__((address_space(4))) * const_u32_ptr;
typedef const float __attribute__((address_space(4))) * const_f32_ptr;

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));

typedef const u32x2 __attribute__((address_space(4))) * const_u32x2_ptr;
typedef const u32x4 __attribute__((address_space(4))) * const_u32x4_ptr;
typedef const u32x8 __attribute__((address_space(4))) * const_u32x8_ptr;
typedef const u32x16 __attribute__((address_space(4))) * const_u32x16_ptr;

// SEG dwords of wave-uniform data held in SGPRs.  The loads are ordinary loads through the
// constant address space from a wave-uniform address, which the compiler turns into
// s_load_dwordxN and tracks itself: it places the s_waitcnt before the first instruction that
// touches a destination register and never reuses those registers while a load is in flight.
// Scalar loads return out of order, so that wait is lgkmcnt(0) and covers every scalar load
// issued before it; the software pipeline (wait for the current buffer, then request the next
// one, then compute) is therefore expressed through data dependences the compiler can see:
// landed() passes the buffer and the address of the next request through one empty asm
// statement, which is the first use of the buffer (the wait goes in front of it) and the
// definition of the address (the next request cannot be moved above it).
template <int SEG>
struct ScalarSeg {
  static constexpr int n16 = SEG / 16, r16 = SEG % 16;
  static constexpr int n8 = r16 / 8, r8 = r16 % 8;
  static constexpr int n4 = r8 / 4, r4 = r8 % 4;
  static constexpr int n2 = r4 / 2, n1 = r4 % 2;
  static_assert(n16 <= 1, "segment longer than 31 dwords");
  u32x16 a16;
  u32x8 a8;
  u32x4 a4;
  u32x2 a2;
  uint32_t a1;

  __device__ __forceinline__ void issue(const_u32_ptr src) {
    if constexpr (n16) a16 = *(const_u32x16_ptr)src;
    if constexpr (n8) a8 = *(const_u32x8_ptr)(src + 16 * n16);
    if constexpr (n4) a4 = *(const_u32x4_ptr)(src + 16 * n16 + 8 * n8);
    if constexpr (n2) a2 = *(const_u32x2_ptr)(src + 16 * n16 + 8 * n8 + 4 * n4);
    if constexpr (n1) a1 = src[16 * n16 + 8 * n8 + 4 * n4 + 2 * n2];
  }
  // The buffer's first use; `next` (the address of the request that follows) is defined here.
  __device__ __forceinline__ void landed(const_u32_ptr& next) {
    if constexpr (n16) asm volatile("" : "+s"(a16), "+s"(next));
    if constexpr (n8) asm volatile("" : "+s"(a8), "+s"(next));
    if constexpr (n4) asm volatile("" : "+s"(a4), "+s"(next));
    if constexpr (n2) asm volatile("" : "+s"(a2), "+s"(next));
    if constexpr (n1) asm volatile("" : "+s"(a1), "+s"(next));
  }
  template <int J>
  __device__ __forceinline__ uint32_t get() const {
    if constexpr (J < 16 * n16) return a16[J];
    else if constexpr (J < 16 * n16 + 8 * n8) return a8[J - 16 * n16];
    else if constexpr (J < 16 * n16 + 8 * n8 + 4 * n4) return a4[J - 16 * n16 - 8 * n8];
    else if constexpr (J < 16 * n16 + 8 * n8 + 4 * n4 + 2 * n2) return a2[J - 16 * n16 - 8 * n8 - 4 * n4];
    else return a1;
  }
};

// Rebuild a wave-uniform address from two readfirstlane halves so that it provably lives
// in SGPRs (64-bit pointer arithmetic is otherwise free to end up on the vector ALU).
__device__ __forceinline__ uint64_t uniform_addr(uint64_t a) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
  return ((uint64_t)hi << 32) | lo;
}

}  // namespace bmx
