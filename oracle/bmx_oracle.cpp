// CPU oracle for the binary-layer hot path of BMXNet (arXiv 1705.09864).
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
// GPU library must compute.  It shares no source, header, table or helper with
// the HIP path and is linked only by the tests, the smoke check and the
// cpu_baseline leg of the benchmark.  It is never a fallback for the product.
//
// The paper's design goal (Sec. 2.2.2, "Training") is that the xnor/popcount
// layers give exactly the output of the ordinary float layers restricted to the
// values -1 and +1.  So the oracle is the ordinary float layer: binarise with
// the sign function (Sec. 1), then a float GEMM / convolution, with none of the
// bit tricks.  All sums of +-1 stay below 2^24 in magnitude, so float
// accumulation is exact and independent of summation order.
//
// Readings of points the paper leaves open (each is also listed in the design
// notes of the repository):
//   * sign(0) = +1, i.e. bit = (x >= 0.0f) as an IEEE compare; NaN gives -1.
//   * packed format: uint64 words, element k is bit (k mod 64) of word k/64,
//     bit 1 <-> +1, bit 0 <-> -1, unused tail bits are 0.
//   * convolution padding: the float image is zero padded first and the sign
//     function is applied afterwards, so padded taps count as +1.
//   * the output is the +-1 dot product; Eq. 2 of the paper relates it to the
//     xnor count: xnor_count = (dot + n) / 2.
//   * alpha (XNOR-Net scale, only named in the abstract) is the mean of |W|
//     over each output row, accumulated in double and rounded once to float.
//   * Eq. 1 "round" is round-half-away-from-zero (C roundf) of the single fp32
//     product (2^k - 1) * x, after clamping x to [0, 1].
//   * k-bit weights (Sec. 2.1 says only that weights follow the same linear
//     quantisation, which Eq. 1 defines on [0, 1]): a weight in [-1, 1] is moved
//     to [0, 1] by u = (w + 1) / 2 (fp32), quantised with Eq. 1 and moved back,
//     w_q = 2 * quantize(u, k) - 1, the affine pair DoReFa-Net wraps around the
//     same quantiser; for k = 1 this is the sign function (threshold at w = 0).
//
// Pins: every function below is checked by tests/test_oracle_*.py against brute
// force, closed forms, invariants and library routines (see those files).

#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

// Sec. 1: binarisation by the sign function, with sign(0) = +1.
inline float sgn(float x) { return (x >= 0.0f) ? 1.0f : -1.0f; }

// Plain float GEMM on already-binarised operands, both stored with K
// contiguous: out[m][n] = sum_k sa[m][k] * sw[n][k]  (Sec. 2.2.2: the float
// layer the binary layer has to match).
void gemm_pm1(const float* sa, const float* sw, int64_t M, int64_t N, int64_t K,
              int32_t* out, int64_t ldo) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    for (int64_t n = 0; n < N; ++n) {
      const float* a = sa + m * K;
      const float* w = sw + n * K;
      float acc = 0.0f;
#pragma omp simd reduction(+ : acc)
      for (int64_t k = 0; k < K; ++k) acc += a[k] * w[k];
      out[m * ldo + n] = (int32_t)acc;
    }
  }
}

}  // namespace

extern "C" {

int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

// Sec. 1: out[i] = sign(x[i]) in {-1, +1}.
void orc_sign(const float* x, int64_t n, float* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = sgn(x[i]);
}

// Sec. 1 / Sec. 2.2.1 (BINARY_WORD): pack 64 binarised elements per word.
// pack_dim = 1: x is [rows, cols], pack along cols -> out[rows][ceil(cols/64)].
// pack_dim = 0: x is [rows, cols] = [K, N], pack along rows -> out[cols][ceil(rows/64)].
// Only the first ceil(K/64) words of each output row are written.
void orc_binarize_pack(const float* x, int64_t rows, int64_t cols, int64_t ldx, int pack_dim,
                       uint64_t* out, int64_t out_ld_words) {
  const int64_t R = pack_dim ? rows : cols;  // packed rows
  const int64_t K = pack_dim ? cols : rows;  // packed length
  const int64_t Kw = (K + 63) / 64;
  for (int64_t r = 0; r < R; ++r) {
    for (int64_t w = 0; w < Kw; ++w) out[r * out_ld_words + w] = 0;
    for (int64_t k = 0; k < K; ++k) {
      const float v = pack_dim ? x[r * ldx + k] : x[k * ldx + r];
      if (v >= 0.0f) out[r * out_ld_words + k / 64] |= (uint64_t)1 << (k % 64);
    }
  }
}

// Inverse of the packed format: element k of row r -> +1.0f / -1.0f.
void orc_unpack_pm1(const uint64_t* p, int64_t rows, int64_t K, int64_t ld_words, float* out) {
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t k = 0; k < K; ++k)
      out[r * K + k] = ((p[r * ld_words + k / 64] >> (k % 64)) & 1) ? 1.0f : -1.0f;
}

// GEMM on packed operands, defined through the float layer (Sec. 2.2.2):
// unpack both to +-1 floats and multiply.  C[m][n] = sum_k a[m][k] * b[n][k].
void orc_xnor_gemm(const uint64_t* A, int64_t lda_w, const uint64_t* B, int64_t ldb_w, int32_t* C,
                   int64_t ldc, int64_t M, int64_t N, int64_t K) {
  std::vector<float> sa((size_t)M * K), sb((size_t)N * K);
  orc_unpack_pm1(A, M, K, lda_w, sa.data());
  orc_unpack_pm1(B, N, K, ldb_w, sb.data());
  gemm_pm1(sa.data(), sb.data(), M, N, K, C, ldc);
}

// XNOR-Net style scale (named in the abstract only; reading stated above):
// alpha[r] = mean_j |w[r][j]|, double accumulation, one rounding to float.
void orc_alpha_mean_abs(const float* w, int64_t rows, int64_t cols, int64_t ldw, float* alpha) {
  for (int64_t r = 0; r < rows; ++r) {
    double s = 0.0;
    for (int64_t j = 0; j < cols; ++j) s += std::fabs((double)w[r * ldw + j]);
    alpha[r] = (float)(s / (double)cols);
  }
}

// QFullyConnected (Sec. 2) on float inputs: binarise activations x [batch, in]
// and weights w [out, in] with the sign function, float GEMM, optional
// per-output scale.  out_i32 and/or out_f32 may be null.
// out_f32[b][o] = (alpha ? alpha[o] : 1) * (float)dot.
void orc_binary_fc(const float* x, int64_t ldx, const float* w, int64_t ldw, const float* alpha,
                   int64_t batch, int64_t in_features, int64_t out_features, int32_t* out_i32,
                   float* out_f32, int64_t ldo) {
  std::vector<float> sx((size_t)batch * in_features), sw((size_t)out_features * in_features);
  for (int64_t b = 0; b < batch; ++b)
    for (int64_t k = 0; k < in_features; ++k) sx[b * in_features + k] = sgn(x[b * ldx + k]);
  for (int64_t o = 0; o < out_features; ++o)
    for (int64_t k = 0; k < in_features; ++k) sw[o * in_features + k] = sgn(w[o * ldw + k]);
  std::vector<int32_t> dot((size_t)batch * out_features);
  gemm_pm1(sx.data(), sw.data(), batch, out_features, in_features, dot.data(), out_features);
  for (int64_t b = 0; b < batch; ++b)
    for (int64_t o = 0; o < out_features; ++o) {
      const int32_t d = dot[b * out_features + o];
      if (out_i32) out_i32[b * ldo + o] = d;
      if (out_f32) out_f32[b * ldo + o] = (alpha ? alpha[o] : 1.0f) * (float)d;
    }
}

// Sec. 3.1: a convolution layer as a GEMM with M = filters, N = batch * output
// pixels, K = kernel_h * kernel_w * input channels.  col is [N_gemm][K] with
// k = (c * KH + kh) * KW + kw; out-of-image taps are 0.0f (ordinary zero
// padding of the float image).
void orc_im2col(const float* x, int64_t N, int64_t C, int64_t H, int64_t W, int64_t KH, int64_t KW,
                int64_t stride, int64_t pad, float* col) {
  const int64_t Ho = (H + 2 * pad - KH) / stride + 1;
  const int64_t Wo = (W + 2 * pad - KW) / stride + 1;
  const int64_t K = C * KH * KW;
  for (int64_t n = 0; n < N; ++n)
    for (int64_t ho = 0; ho < Ho; ++ho)
      for (int64_t wo = 0; wo < Wo; ++wo) {
        float* dst = col + ((n * Ho + ho) * Wo + wo) * K;
        for (int64_t c = 0; c < C; ++c)
          for (int64_t kh = 0; kh < KH; ++kh)
            for (int64_t kw = 0; kw < KW; ++kw) {
              const int64_t h = ho * stride - pad + kh;
              const int64_t w = wo * stride - pad + kw;
              const bool in = (h >= 0 && h < H && w >= 0 && w < W);
              dst[(c * KH + kh) * KW + kw] = in ? x[((n * C + c) * H + h) * W + w] : 0.0f;
            }
      }
}

// QConvolution (Sec. 2, Sec. 3.1): zero-padded float im2col, then the sign
// function on every element (so padding becomes +1), then the float GEMM
// against sign(weights), optional per-output-channel scale.  x is NCHW, w is
// OIHW, outputs are NCHW [N, O, Ho, Wo]; out_i32 and/or out_f32 may be null.
void orc_binary_conv2d(const float* x, int64_t N, int64_t C, int64_t H, int64_t W, const float* w,
                       int64_t O, int64_t KH, int64_t KW, int64_t stride, int64_t pad,
                       const float* alpha, int32_t* out_i32, float* out_f32) {
  const int64_t Ho = (H + 2 * pad - KH) / stride + 1;
  const int64_t Wo = (W + 2 * pad - KW) / stride + 1;
  const int64_t K = C * KH * KW;
  const int64_t P = N * Ho * Wo;
  std::vector<float> col((size_t)P * K), sw((size_t)O * K);
  orc_im2col(x, N, C, H, W, KH, KW, stride, pad, col.data());
  for (size_t i = 0; i < col.size(); ++i) col[i] = sgn(col[i]);
  for (size_t i = 0; i < sw.size(); ++i) sw[i] = sgn(w[i]);
  std::vector<int32_t> dot((size_t)O * P);
  gemm_pm1(sw.data(), col.data(), O, P, K, dot.data(), P);  // [O][N*Ho*Wo]
  for (int64_t n = 0; n < N; ++n)
    for (int64_t o = 0; o < O; ++o)
      for (int64_t p = 0; p < Ho * Wo; ++p) {
        const int32_t d = dot[o * P + n * Ho * Wo + p];
        const int64_t idx = (n * O + o) * Ho * Wo + p;
        if (out_i32) out_i32[idx] = d;
        if (out_f32) out_f32[idx] = (alpha ? alpha[o] : 1.0f) * (float)d;
      }
}

// The same layer written as the direct nested-loop convolution (no im2col, no
// GEMM): used only to pin orc_binary_conv2d from a second, independent side.
void orc_binary_conv2d_direct(const float* x, int64_t N, int64_t C, int64_t H, int64_t W,
                              const float* w, int64_t O, int64_t KH, int64_t KW, int64_t stride,
                              int64_t pad, int32_t* out_i32) {
  const int64_t Ho = (H + 2 * pad - KH) / stride + 1;
  const int64_t Wo = (W + 2 * pad - KW) / stride + 1;
  for (int64_t n = 0; n < N; ++n)
    for (int64_t o = 0; o < O; ++o)
      for (int64_t ho = 0; ho < Ho; ++ho)
        for (int64_t wo = 0; wo < Wo; ++wo) {
          double acc = 0.0;
          for (int64_t c = 0; c < C; ++c)
            for (int64_t kh = 0; kh < KH; ++kh)
              for (int64_t kw = 0; kw < KW; ++kw) {
                const int64_t h = ho * stride - pad + kh;
                const int64_t ww = wo * stride - pad + kw;
                const float xv =
                    (h >= 0 && h < H && ww >= 0 && ww < W) ? x[((n * C + c) * H + h) * W + ww] : 0.0f;
                acc += (double)sgn(xv) * (double)sgn(w[((o * C + c) * KH + kh) * KW + kw]);
              }
          out_i32[((n * O + o) * Ho + ho) * Wo + wo] = (int32_t)acc;
        }
}

// Eq. 1: quantize(x, k) = round((2^k - 1) * x) / (2^k - 1) for x in [0, 1].
// q_int[i] receives the integer level round((2^k - 1) * x) in [0, 2^k - 1],
// q_val[i] (double, may be null) the quantised real value.
void orc_quantize(const float* x, int64_t n, int bits, int32_t* q_int, double* q_val) {
  const float levels = (float)((1u << bits) - 1u);
  for (int64_t i = 0; i < n; ++i) {
    float v = x[i];
    v = (v < 0.0f) ? 0.0f : (v > 1.0f ? 1.0f : v);
    const float t = levels * v;  // one fp32 product
    const int32_t q = (int32_t)std::round(t);
    if (q_int) q_int[i] = q;
    if (q_val) q_val[i] = (double)q / (double)levels;
  }
}

// k-bit activations (Eq. 1) times 1-bit sign weights (Sec. 2.1 keeps quantised
// values as floats and uses the standard dot product; so does this):
//   out_f64[m][n] = sum_k quantize(a[m][k], bits) * sign(w[n][k])   (double)
//   S[m][n]       = sum_k level(a[m][k]) * sign(w[n][k])            (exact integer)
//   out_f32[m][n] = (float)S / (float)(2^bits - 1)
// Any of the three outputs may be null.
void orc_quant_gemm(const float* a, int64_t lda, int bits_a, const float* w, int64_t ldw, int64_t M,
                    int64_t N, int64_t K, int32_t* S, double* out_f64, float* out_f32, int64_t ldo) {
  std::vector<int32_t> q((size_t)M * K);
  std::vector<double> qv((size_t)M * K);
  for (int64_t m = 0; m < M; ++m) orc_quantize(a + m * lda, K, bits_a, &q[m * K], &qv[m * K]);
  std::vector<float> sw((size_t)N * K);
  for (int64_t n = 0; n < N; ++n)
    for (int64_t k = 0; k < K; ++k) sw[n * K + k] = sgn(w[n * ldw + k]);
  const float levels = (float)((1u << bits_a) - 1u);
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double accf = 0.0;
      int64_t acci = 0;
      for (int64_t k = 0; k < K; ++k) {
        accf += qv[m * K + k] * (double)sw[n * K + k];
        acci += (int64_t)q[m * K + k] * (int64_t)sw[n * K + k];
      }
      if (out_f64) out_f64[m * ldo + n] = accf;
      if (S) S[m * ldo + n] = (int32_t)acci;
      if (out_f32) out_f32[m * ldo + n] = (float)acci / levels;
    }
}

// k-bit activations times k-bit weights (reading above):
//   out_f64[m][n] = sum_k quantize(a[m][k], bits_a) * (2 * quantize((w[n][k] + 1) / 2, bits_w) - 1)
//   S[m][n]       = sum_k level_a * (2 * level_w - (2^bits_w - 1))      (exact integer)
//   out_f32[m][n] = (float)S / (float)((2^bits_a - 1) * (2^bits_w - 1))
void orc_quant_gemm_kw(const float* a, int64_t lda, int bits_a, const float* w, int64_t ldw, int bits_w,
                       int64_t M, int64_t N, int64_t K, int32_t* S, double* out_f64, float* out_f32,
                       int64_t ldo) {
  std::vector<int32_t> qa((size_t)M * K), qw((size_t)N * K);
  std::vector<double> va((size_t)M * K), vw((size_t)N * K);
  for (int64_t m = 0; m < M; ++m) orc_quantize(a + m * lda, K, bits_a, &qa[m * K], &va[m * K]);
  std::vector<float> u((size_t)K);
  for (int64_t n = 0; n < N; ++n) {
    for (int64_t k = 0; k < K; ++k) u[k] = (w[n * ldw + k] + 1.0f) * 0.5f;
    orc_quantize(u.data(), K, bits_w, &qw[n * K], &vw[n * K]);
    for (int64_t k = 0; k < K; ++k) vw[n * K + k] = 2.0 * vw[n * K + k] - 1.0;
  }
  const int64_t La = (1 << bits_a) - 1, Lw = (1 << bits_w) - 1;
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int64_t n = 0; n < N; ++n) {
      double accf = 0.0;
      int64_t acci = 0;
      for (int64_t k = 0; k < K; ++k) {
        accf += va[m * K + k] * vw[n * K + k];
        acci += (int64_t)qa[m * K + k] * (2 * (int64_t)qw[n * K + k] - Lw);
      }
      if (out_f64) out_f64[m * ldo + n] = accf;
      if (S) S[m * ldo + n] = (int32_t)acci;
      if (out_f32) out_f32[m * ldo + n] = (float)acci / (float)(La * Lw);
    }
}

}  // extern "C"
