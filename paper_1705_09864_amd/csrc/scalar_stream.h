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

// SEG dwords of wave-uniform data held in SGPRs, fetched with explicit scalar loads.
// Scalar loads return out of order, so the only usable wait is lgkmcnt(0); issuing the
// loads and waiting for them are therefore separate, explicitly placed steps: wait for the
// current buffer, then issue the next one, then compute.  The loads are written as
// volatile asm so that the compiler neither tracks them (it would merge both buffers into
// one wait) nor moves them.
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

  // `tie` is an accumulator the following VALU work depends on: threading it through the
  // first load keeps that work behind the issue point.
  __device__ __forceinline__ void issue(const_u32_ptr src, int& tie) {
    asm volatile("" : "+v"(tie));
    if constexpr (n16) asm volatile("s_load_dwordx16 %0, %1, 0x0" : "=s"(a16) : "s"(src));
    if constexpr (n8) asm volatile("s_load_dwordx8 %0, %1, %2" : "=s"(a8) : "s"(src), "i"(64 * n16));
    if constexpr (n4)
      asm volatile("s_load_dwordx4 %0, %1, %2" : "=s"(a4) : "s"(src), "i"(64 * n16 + 32 * n8));
    if constexpr (n2)
      asm volatile("s_load_dwordx2 %0, %1, %2" : "=s"(a2)
                   : "s"(src), "i"(64 * n16 + 32 * n8 + 16 * n4));
    if constexpr (n1)
      asm volatile("s_load_dword %0, %1, %2" : "=s"(a1)
                   : "s"(src), "i"(64 * n16 + 32 * n8 + 16 * n4 + 8 * n2));
    asm volatile("" : "+v"(tie));
  }
  // All outstanding scalar loads have landed after this; every piece is threaded through
  // an asm statement so that no use can be placed before the wait.
  __device__ __forceinline__ void wait() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if constexpr (n16) asm volatile("" : "+s"(a16));
    if constexpr (n8) asm volatile("" : "+s"(a8));
    if constexpr (n4) asm volatile("" : "+s"(a4));
    if constexpr (n2) asm volatile("" : "+s"(a2));
    if constexpr (n1) asm volatile("" : "+s"(a1));
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
