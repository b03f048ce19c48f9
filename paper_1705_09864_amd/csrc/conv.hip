// Implicit-GEMM binary convolution on the channel-packed image (VALU integer bound).
// Paper: Sec. 3.1 (M = filters, N = batch * output pixels, K = kh * kw * C); the
// im2col matrix is never formed: each lane gathers its taps from Xp [N][H][W][Cw].
#include "bmx_internal.h"

namespace bmx {

// Lanes span output pixels (coalesced NCHW stores), the filter row is wave-uniform.
// A tap outside the image reads as "all real channels = +1": the float image is zero
// padded before the sign function and sign(0) = +1.
__global__ void __launch_bounds__(256)
binary_conv2d_kernel(const uint64_t* __restrict__ Xp, int N, int C, int H, int W,
                     const uint64_t* __restrict__ Wp, int O, int KH, int KW, int stride, int pad,
                     int Ho, int Wo, int Cw, const float* __restrict__ alpha,
                     int32_t* __restrict__ out_i32, float* __restrict__ out_f32) {
  const int64_t P = (int64_t)N * Ho * Wo;
  const int64_t p = (int64_t)blockIdx.x * 64 + (threadIdx.x & 63);
  const int o = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (p >= P || o >= O) return;
  const int wo = (int)(p % Wo);
  const int ho = (int)((p / Wo) % Ho);
  const int n = (int)(p / ((int64_t)Wo * Ho));
  const uint64_t tail = (C % 64) ? (((uint64_t)1 << (C % 64)) - 1) : ~(uint64_t)0;
  const uint64_t* wrow = Wp + (int64_t)o * KH * KW * Cw;
  int pc = 0;
  for (int kh = 0; kh < KH; ++kh) {
    const int h = ho * stride - pad + kh;
    for (int kw = 0; kw < KW; ++kw) {
      const int w = wo * stride - pad + kw;
      const bool in = (h >= 0 && h < H && w >= 0 && w < W);
      const uint64_t* xp = Xp + (((int64_t)n * H + h) * W + w) * Cw;
      const uint64_t* wp = wrow + (kh * KW + kw) * Cw;
      for (int cw = 0; cw < Cw; ++cw) {
        const uint64_t ones = (cw == Cw - 1) ? tail : ~(uint64_t)0;
        const uint64_t xv = in ? xp[cw] : ones;
        pc += __popcll(xv ^ wp[cw]);
      }
    }
  }
  const int dot = C * KH * KW - 2 * pc;
  const int64_t idx = (((int64_t)n * O + o) * Ho + ho) * Wo + wo;
  if (out_i32) out_i32[idx] = dot;
  else out_f32[idx] = (alpha ? alpha[o] : 1.0f) * (float)dot;
}

hipError_t launch_binary_conv2d(const uint64_t* Xp, int N, int C, int H, int W, const uint64_t* Wp,
                                int O, int KH, int KW, int stride, int pad, const float* alpha,
                                int32_t* out_i32, float* out_f32, hipStream_t s) {
  const int Ho = (H + 2 * pad - KH) / stride + 1;
  const int Wo = (W + 2 * pad - KW) / stride + 1;
  const int64_t P = (int64_t)N * Ho * Wo;
  dim3 grid((unsigned)ceil_div(P, 64), (unsigned)ceil_div(O, 4));
  hipLaunchKernelGGL(binary_conv2d_kernel, grid, dim3(256), 0, s, Xp, N, C, H, W, Wp, O, KH, KW,
                     stride, pad, Ho, Wo, (int)words_for(C), alpha, out_i32, out_f32);
  return hipGetLastError();
}

}  // namespace bmx
