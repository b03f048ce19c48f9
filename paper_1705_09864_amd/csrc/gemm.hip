// xor + popcount GEMM kernels on packed operands (VALU integer bound).
// Paper: Sec. 2.2.1 (xnor GEMM on packed words), Sec. 2.2.2 / Eq. 2 (output range).
#include "bmx_internal.h"

namespace bmx {

// C[m][n] = K - 2 * sum_i popcount(A[m][i] ^ B[n][i]).
// Lanes span n (coalesced C stores); the A row is wave-uniform.
__global__ void __launch_bounds__(256)
xnor_gemm_kernel(const uint64_t* __restrict__ A, int64_t lda_w, const uint64_t* __restrict__ B,
                 int64_t ldb_w, int M, int N, int K, int Kw, const float* __restrict__ alpha_n,
                 int32_t* __restrict__ C_i32, float* __restrict__ C_f32, int64_t ldc) {
  const int n = blockIdx.x * 64 + (threadIdx.x & 63);
  const int m = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (m >= M || n >= N) return;
  const uint64_t* a = A + (int64_t)m * lda_w;
  const uint64_t* b = B + (int64_t)n * ldb_w;
  int pc = 0;
  for (int i = 0; i < Kw; ++i) pc += __popcll(a[i] ^ b[i]);
  const int dot = K - 2 * pc;
  if (C_i32) C_i32[(int64_t)m * ldc + n] = dot;
  else C_f32[(int64_t)m * ldc + n] = (alpha_n ? alpha_n[n] : 1.0f) * (float)dot;
}

hipError_t launch_xnor_gemm(const uint64_t* A, int64_t lda_w, const uint64_t* B, int64_t ldb_w,
                            int M, int N, int K, const float* alpha_n, int32_t* C_i32, float* C_f32,
                            int64_t ldc, hipStream_t s) {
  dim3 grid((unsigned)ceil_div(N, 64), (unsigned)ceil_div(M, 4));
  hipLaunchKernelGGL(xnor_gemm_kernel, grid, dim3(256), 0, s, A, lda_w, B, ldb_w, M, N, K,
                     (int)words_for(K), alpha_n, C_i32, C_f32, ldc);
  return hipGetLastError();
}

// Bit-plane GEMM: S[m][n] = 2 * sum_p 2^p popcount(plane_p[m] & Wb[n]) - rowsum[m].
__global__ void __launch_bounds__(256)
plane_gemm_kernel(const uint64_t* __restrict__ planes, int bits, const int32_t* __restrict__ rowsum,
                  const uint64_t* __restrict__ Wb, int M, int N, int Kw, int32_t* __restrict__ S,
                  float* __restrict__ out_f32, int64_t ldo) {
  const int n = blockIdx.x * 64 + (threadIdx.x & 63);
  const int m = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (m >= M || n >= N) return;
  const uint64_t* b = Wb + (int64_t)n * Kw;
  int acc = 0;
  for (int p = 0; p < bits; ++p) {
    const uint64_t* a = planes + ((int64_t)p * M + m) * Kw;
    int pc = 0;
    for (int i = 0; i < Kw; ++i) pc += __popcll(a[i] & b[i]);
    acc += pc << p;
  }
  const int s = 2 * acc - rowsum[m];
  if (S) S[(int64_t)m * ldo + n] = s;
  if (out_f32) out_f32[(int64_t)m * ldo + n] = (float)s / (float)((1u << bits) - 1u);
}

hipError_t launch_plane_gemm(const uint64_t* planes, int bits, const int32_t* rowsum,
                             const uint64_t* Wb, int M, int N, int K, int32_t* S, float* out_f32,
                             int64_t ldo, hipStream_t s) {
  dim3 grid((unsigned)ceil_div(N, 64), (unsigned)ceil_div(M, 4));
  hipLaunchKernelGGL(plane_gemm_kernel, grid, dim3(256), 0, s, planes, bits, rowsum, Wb, M, N,
                     (int)words_for(K), S, out_f32, ldo);
  return hipGetLastError();
}

}  // namespace bmx
