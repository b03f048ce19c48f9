// Binary fully connected layer for problems of a few microseconds of work or less, in one launch.
// Paper: Sec. 2 (QFullyConnected: binarise the input, xnor GEMM against the packed weights,
// optional scale), Sec. 2.2.1 / 2.2.2 (Eq. 2): out[m][n] = K - 2 * popcount(x_bits[m] xor W[n]).
//
// A layer this small (64 x 512 -> 256: 13 ns of arithmetic) is two launches on the general path,
// pack then GEMM, each a launch plus a chain of trips to memory, about 3.5 us apiece.  Here a
// workgroup takes one batch row: its waves turn the row's fp32 values into sign bits in LDS (one
// coalesced load and one ballot per 64 values), and thread t then produces output features
// t, t + 256, ... with xor + popcount of the row's words against the feature's packed weights,
// whose first words it requested before the row was packed.  The weights are read once per
// batch row (from L2 after the first), which is why the launcher takes only small layers.
#include "bmx_internal.h"

namespace bmx {

namespace {

constexpr int kAhead = 8;  // weight words a thread requests ahead of the pack

__global__ void __launch_bounds__(256)
fc_small_kernel(const float* __restrict__ x, int64_t ldx, const uint64_t* __restrict__ Wp, int64_t ldw_w,
                const float* __restrict__ alpha, int K, int Kw, int N, int32_t* __restrict__ out_i32,
                float* __restrict__ out_f32, int64_t ldo) {
  extern __shared__ uint64_t row[];  // the batch row's Kw words of sign bits
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = blockIdx.x;
  // this thread's first output feature: its first weight words, requested first of all
  const int n_first = min((int)threadIdx.x, N - 1);
  uint64_t wfirst[kAhead];
#pragma unroll
  for (int w = 0; w < kAhead; ++w) wfirst[w] = Wp[(int64_t)n_first * ldw_w + min(w, Kw - 1)];
  // sign bits of the row: wave v takes words v, v + 4, ..., four at a time so that their loads
  // are in flight together; values past K count as negative (bit 0, like the packed weights' tail)
  const float* xr = x + (int64_t)m * ldx;
  for (int w0 = wave; w0 < Kw; w0 += 16) {
    float v[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = 64 * (w0 + 4 * i) + lane;
      v[i] = k < K ? xr[k] : -1.0f;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint64_t bits = __ballot(v[i] >= 0.0f);
      if (lane == 0 && w0 + 4 * i < Kw) row[w0 + 4 * i] = bits;
    }
  }
  __syncthreads();
  for (int n = threadIdx.x; n < N; n += 256) {
    const uint64_t* wr = Wp + (int64_t)n * ldw_w;
    int pc = 0;
    if (n == (int)threadIdx.x) {
#pragma unroll
      for (int w = 0; w < kAhead; ++w)
        if (w < Kw) pc += __popcll(row[w] ^ wfirst[w]);
      for (int w = kAhead; w < Kw; ++w) pc += __popcll(row[w] ^ wr[w]);
    } else {
      for (int w = 0; w < Kw; ++w) pc += __popcll(row[w] ^ wr[w]);
    }
    const int dot = K - 2 * pc;
    if (out_i32) out_i32[(int64_t)m * ldo + n] = dot;
    else out_f32[(int64_t)m * ldo + n] = (alpha ? alpha[n] : 1.0f) * (float)dot;
  }
}

}  // namespace

int fc_small = 0;  // 1 = never (measurements and tests of the general path on small layers)

// Takes layers whose whole weight matrix is at most 64 words per thread of a workgroup and whose
// rows fit 8 KB of LDS; false otherwise.
bool launch_fc_small(const float* x, int64_t ldx, const uint64_t* Wp, int64_t ldw_w, const float* alpha, int batch,
                     int in_features, int out_features, int32_t* out_i32, float* out_f32, int64_t ldo,
                     hipStream_t s, hipError_t* err) {
  const int64_t Kw = words_for(in_features);
  // (a GEMM engine pinned through the tuning hook is what the caller wants to run)
  if (fc_small == 1 || gemm_engine != 0 || Kw > 1024 || (int64_t)out_features * Kw > 256 * 64 || batch > 4096) return false;
  note_kernel("fc_small_kernel grid %d x 256", batch);
  hipLaunchKernelGGL(fc_small_kernel, dim3((unsigned)batch), dim3(256), (size_t)Kw * 8, s, x, ldx, Wp, ldw_w, alpha,
                     in_features, (int)Kw, out_features, out_i32, out_f32, ldo);
  *err = hipGetLastError();
  return true;
}

}  // namespace bmx
