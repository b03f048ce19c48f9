// Internal launcher declarations shared by the translation units of libbmx.
// Every launcher assumes its arguments were validated by the C-ABI layer
// (bmx_api.hip) and returns hipGetLastError() after enqueueing its kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bmx {

__host__ __device__ static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
// Division of a 32-bit unsigned by a runtime constant as multiply-high + shifts.
struct FastDiv {
  uint32_t mul, sh1, sh2;
};
FastDiv make_fast_div(uint32_t d);
// q = n / d for 0 <= n < 2^32 by multiply-high (Granlund-Montgomery round-up method).
__device__ static inline uint32_t fast_div(uint32_t n, FastDiv f) {
  const uint32_t t = __umulhi(f.mul, n);
  return (t + ((n - t) >> f.sh1)) >> f.sh2;
}

__host__ __device__ static inline int64_t words_for(int64_t k) { return (k + 63) / 64; }

// Name (with template arguments and launch shape) of the kernel the calling thread launched
// last: what bmx_last_kernel() reports, so that measurements label themselves.
void note_kernel(const char* fmt, ...) __attribute__((format(printf, 1, 2)));

// Packed rows that feed the scalar side of the GEMM kernel are zero padded to whole
// 32-dword chunks, so that every chunk of a row can be fetched with two 64-byte scalar loads.
__host__ __device__ static inline int64_t padded_words(int64_t K) {
  return ceil_div(words_for(K), 16) * 16;
}

// Packed convolution weights: filter o is row o of a matrix with kwords = KH * KW * ceil(C/64)
// data words per row, zero padded to whole register chunks of the GEMM kernel.  The chunk is
// 24 or 32 dwords, whichever wastes less padding (3 x 3 kernels over a multiple of 256
// channels fit 24 exactly).
__host__ __device__ static inline int conv_weight_chunk_dwords(int64_t kwords) {
  const int64_t p24 = ceil_div(2 * kwords, 24) * 24, p32 = ceil_div(2 * kwords, 32) * 32;
  return p24 < p32 ? 24 : 32;
}
__host__ __device__ static inline int64_t conv_weight_bits_words(int64_t kwords) {
  const int ch = conv_weight_chunk_dwords(kwords);
  return ceil_div(2 * kwords, ch) * ch / 2;
}
// For the K the short-K matrix-core convolution kernel takes (the list below) a row carries,
// behind its chunk-padded bits, two more words: the float K - 2 * popcount(filter) in the first
// dword, zeros after it (the kernel's epilogue constant, computed once with the offline weight
// pack of Sec. 2.2.3; rows stay a whole number of 16 bytes).
__host__ __device__ static inline bool conv_weight_short_k(int64_t kwords) {
  return kwords == 9 || kwords == 18 || kwords == 25 || kwords == 27 || kwords == 36 || kwords == 49 || kwords == 50;
}
__host__ __device__ static inline int64_t conv_weight_row_words(int64_t kwords) {
  return conv_weight_bits_words(kwords) + (conv_weight_short_k(kwords) ? 2 : 0);
}

// pack.hip -------------------------------------------------------------------
// Row pack: out[r][w] bit j = (x[r*ldx + 64w + j] >= 0), K contiguous in x.
hipError_t launch_pack_rows(const float* x, int64_t rows, int64_t cols, int64_t ldx, uint64_t* out,
                            int64_t out_ld, hipStream_t s);
// Strided pack of `batch` matrices stored [K][ncol] (row stride ldx, matrix stride
// batch_stride): out[b][n][w] bit j = (x[b][64w + j][n] >= 0); out row stride out_ld,
// matrix stride ncol*out_ld.  Serves pack_dim = 0 and the NCHW channel pack.
hipError_t launch_unpack_pm1(const uint64_t* bits, int64_t rows, int64_t K, int64_t ld_words, float* out,
                             int64_t ldo, hipStream_t s);
// Rows of ceil(K/32) 32-bit words, ld_dw apart -> rows of ceil(K/64) 64-bit words, out_ld apart.
hipError_t launch_widen_words32(const uint32_t* in, int64_t rows, int64_t K, int64_t ld_dw, uint64_t* out,
                                int64_t out_ld, hipStream_t s);
hipError_t launch_pack_strided(const float* x, int64_t batch, int64_t K, int64_t ncol, int64_t ldx,
                               int64_t batch_stride, uint64_t* out, int64_t out_ld, hipStream_t s);
// NCHW channel pack into the halo-padded layout xp [N][H+2*pad][W+2*pad][Cw]; the halo is
// filled with the word "all real channels = +1".
// (thr: per-channel threshold the value is compared with, null = 0)
hipError_t launch_pack_nchw_thr(const float* x, int N, int C, int H, int W, int pad, const float* thr,
                                uint64_t* xp, hipStream_t s);
hipError_t launch_pack_nchw(const float* x, int N, int C, int H, int W, int pad, uint64_t* xp,
                            hipStream_t s);
hipError_t launch_pack_conv_weights(const float* w, int O, int C, int KH, int KW, uint64_t* Wp,
                                    hipStream_t s);
hipError_t launch_alpha_mean_abs(const float* w, int64_t rows, int64_t cols, int64_t ldw,
                                 float* alpha, hipStream_t s);
// Row pack into rows of out_ld words where every word up to out_ld is written (zeros past
// ceil(cols/64)): the chunk-padded activation rows of the FC layer.
hipError_t launch_pack_rows_padded(const float* x, int64_t rows, int64_t cols, int64_t ldx,
                                   uint64_t* out, int64_t out_ld, hipStream_t s);
// Eq. 1 quantise + bit-plane pack: plane p of row m is row m * bits + p of `planes`
// (row stride ld_words, zero padded to it); rowsum[m] = sum_k q[m][k].  With wrows > 0 the
// same launch also sign-packs w [wrows, K] (row stride ldw) into wbits (row stride wb_ld).
hipError_t launch_quant_pack(const float* a, int64_t M, int64_t K, int64_t lda, int bits,
                             uint64_t* planes, int64_t ld_words, int32_t* rowsum, const float* w,
                             int64_t wrows, int64_t ldw, uint64_t* wbits, int64_t wb_ld,
                             hipStream_t s, bool affine = false);
hipError_t launch_quant_combine(const int32_t* T, int64_t M, int64_t N, int bw, float denom, int32_t* S,
                                float* out, int64_t ldo, hipStream_t s);

// probe.hip: register-only xor + popcount chain, for the peak and clock measurement hook.
hipError_t launch_probe_valu(int workgroups, int iters, unsigned long long* out3, hipStream_t s);

// gemm.hip -------------------------------------------------------------------
// out = K - 2*popcount(A ^ B); exactly one of C_i32 / C_f32 / C_bits non-null;
// C_f32[m][n] = (alpha_n ? alpha_n[n] : 1) * float(dot).
// A is row-major with lda_dw dwords per row.  a_padded: every row is readable and zero up
// to a multiple of 32 dwords (workspace copies); otherwise only ceil(K/64) words per row
// are touched.
// C_bits (instead of C_i32 / C_f32): packed (alpha_n[n] * float(dot) >= thr_n[n]), thr_n null
// = 0, ldc words per row.
hipError_t launch_xnor_gemm(const uint32_t* A, bool a_padded, int64_t lda_dw, const uint64_t* B,
                            int64_t ldb_w, int M, int N, int K, const float* alpha_n, int32_t* C_i32,
                            float* C_f32, uint64_t* C_bits, const float* thr_n, int64_t ldc, hipStream_t s,
                            bool as_count = false);  // as_count: C_i32 = (dot + K) / 2, the xnor count of Eq. 2
// gemm_mfma.hip: the same product on the int8 matrix cores (operands expanded from bits in
// registers).  Returns false when it does not take the problem (engine choice, alignment).
bool launch_xnor_gemm_mfma(const uint64_t* A, int64_t lda_w, const uint64_t* B, int64_t ldb_w, int M,
                           int N, int K, const float* alpha_n, int32_t* C_i32, float* C_f32,
                           uint64_t* C_bits, const float* thr_n, int64_t ldc, hipStream_t s, hipError_t* err,
                           bool as_count = false);
// gemm_fp4.hip: the same products with 64 x 64 of C per wave, operands staged through LDS by
// the load unit, K split over the waves of a workgroup (FP4 only; planes = 1 with rowsum null is
// the xnor form, otherwise the plane form with 1 or 2 planes).  Returns false when it does not
// take the problem.
bool launch_gemm_fp4(const uint64_t* A, int64_t lda_w, int planes, const int32_t* rowsum, const uint64_t* B,
                     int64_t ldb_w, int M, int N, int K, const float* alpha_n, int32_t* C_i32, float* C_f32,
                     uint64_t* C_bits, const float* thr_n, int64_t ldc, bool as_count, hipStream_t s,
                     hipError_t* err);
bool launch_conv_fp4(const uint64_t* Xp, int Nimg, int C, int H, int W, const uint64_t* Wp, int O, int KH, int KW,
                     int stride, int pad, const float* alpha, int32_t* out_i32, float* out_f32, hipStream_t s,
                     hipError_t* err);
extern int gemm_fp4_split, gemm_fp4_half, gemm_fp4_band, gemm_fp4_tall;
// fc_small.hip: the whole fully connected layer (sign bits of the fp32 input, xor + popcount,
// scale) in one launch, for layers too small to be worth two; false when the layer is not
// small enough (nothing launched then).
bool launch_fc_small(const float* x, int64_t ldx, const uint64_t* Wp, int64_t ldw_w, const float* alpha, int batch,
                     int in_features, int out_features, int32_t* out_i32, float* out_f32, int64_t ldo,
                     hipStream_t s, hipError_t* err);
extern int fc_small;
bool launch_plane_gemm_mfma(const uint64_t* planes_rows, int64_t lda_w, int bits, const int32_t* rowsum,
                            const uint64_t* Wb, int64_t ldb_w, int M, int N, int K, int32_t* S_out,
                            float* out_f32, int64_t ldo, hipStream_t s, hipError_t* err);
bool launch_conv_mfma(const uint64_t* Xp, int Nimg, int C, int H, int W, const uint64_t* Wp, int O, int KH,
                      int KW, int stride, int pad, const float* alpha, int32_t* out_i32, float* out_f32,
                      hipStream_t s, hipError_t* err);
// conv_mfma.hip: the convolution on the FP4 matrix cores with the expanded filters of a
// workgroup in LDS (K as conv_weight_short_k lists).  Returns false outside its domain.  With out_bits
// the result leaves as the packed image of the next convolution (halo out_pad, written too):
// bit o = (alpha[o] * dot >= thr[o]), thr null = 0.
bool conv_mfma_ws_takes(int Nimg, int C, int H, int W, int O, int KH, int KW, int stride, int pad,
                        int out_pad);  // its domain, the 16-byte alignment of Wp aside
bool launch_conv_mfma_ws(const uint64_t* Xp, int Nimg, int C, int H, int W, const uint64_t* Wp, int O,
                         int KH, int KW, int stride, int pad, const float* alpha, int32_t* out_i32,
                         float* out_f32, uint64_t* out_bits, const float* thr, int out_pad, hipStream_t s,
                         hipError_t* err);
extern int gemm_engine, gemm_mfma_ksplit, gemm_mfma_tile, conv_filters_per_wave, conv_path, conv_ws_x4;
// S = 2*sum_p 2^p pc(plane_p & wb) - rowsum; out_f32 = float(S) / float(2^bits - 1).
// planes_rows as written by launch_quant_pack (lda_dw dwords per row, chunk padded).
hipError_t launch_plane_gemm(const uint32_t* planes_rows, int64_t lda_dw, int bits,
                             const int32_t* rowsum, const uint64_t* Wb, int64_t ldb_w, int M, int N,
                             int K, int32_t* S, float* out_f32, int64_t ldo, hipStream_t s);

// The same convolution on the GEMM kernel (filters = A rows streamed through SGPRs, im2col
// rows gathered per chunk): for K that does not fit the stationary kernel or grids with too
// few pixel groups for it.
hipError_t launch_conv_gemm(const uint64_t* Xp, int Nimg, int C, int H, int W, const uint64_t* Wp,
                            int O, int KH, int KW, int stride, int pad, const float* alpha,
                            int32_t* out_i32, float* out_f32, hipStream_t s);

// conv.hip -------------------------------------------------------------------
// Implicit-GEMM convolution on the halo-padded channel-packed image from launch_pack_nchw.
hipError_t launch_binary_conv2d(const uint64_t* Xp, int N, int C, int H, int W, const uint64_t* Wp,
                                int O, int KH, int KW, int stride, int pad, const float* alpha,
                                int32_t* out_i32, float* out_f32, hipStream_t s);

}  // namespace bmx
