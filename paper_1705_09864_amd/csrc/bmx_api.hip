// C-ABI layer of libbmx: host-side argument validation and dispatch.
// Every check happens before the first launch, so an error return means that no kernel
// ran and no output byte was written.  The contract of each call is in include/bmx.h.
#include "../../include/bmx.h"
#include "bmx_internal.h"

#include <cstdarg>
#include <cstdio>
#include <mutex>

// Scratch memory of bmx_binary_fc_static, the entry point for callers that cannot allocate: one
// copy per GPU the library runs on, held until the process ends.  In host code this name is only
// a handle for hipGetSymbolAddress, never an address to hand to a kernel.
#define BMX_STATIC_SCRATCH_BYTES (4u << 20)
static __device__ __align__(256) unsigned char scratch[BMX_STATIC_SCRATCH_BYTES];

namespace {

constexpr int64_t kMaxK = (int64_t)1 << 24;  // float(dot) stays exact below this

inline bool misaligned(const void* p, size_t a) { return ((uintptr_t)p % a) != 0; }
inline size_t round256(size_t b) { return (b + 255) & ~(size_t)255; }
inline int hip_status(hipError_t e) { return e == hipSuccess ? BMX_OK : BMX_ERR_HIP; }

struct ConvGeom {
  int Ho, Wo, Cw;
};

int conv_check(int N, int C, int H, int W, int O, int KH, int KW, int stride, int pad,
               ConvGeom* g) {
  if (N < 0 || C <= 0 || H <= 0 || W <= 0 || O < 0) return BMX_ERR_SHAPE;
  if (KH != KW || !(KH == 1 || KH == 3 || KH == 5 || KH == 7)) return BMX_ERR_UNSUPPORTED;
  if (!(stride == 1 || stride == 2)) return BMX_ERR_UNSUPPORTED;
  if (pad < 0 || pad >= KH) return BMX_ERR_UNSUPPORTED;
  if ((int64_t)C * KH * KW >= kMaxK) return BMX_ERR_SHAPE;
  if (H + 2 * pad < KH || W + 2 * pad < KW) return BMX_ERR_SHAPE;
  g->Ho = (H + 2 * pad - KH) / stride + 1;
  g->Wo = (W + 2 * pad - KW) / stride + 1;
  g->Cw = (int)bmx::words_for(C);
  // (filters: the one-thread-per-output kernel puts four of them on a workgroup of grid.y)
  if ((int64_t)N * g->Ho * g->Wo >= ((int64_t)1 << 31) || N > 65535 || O > 4 * 65535)
    return BMX_ERR_SHAPE;
  if ((int64_t)(H + 2 * pad) * (W + 2 * pad) >= ((int64_t)1 << 31)) return BMX_ERR_SHAPE;
  return BMX_OK;
}

// 64-bit row length (even: 16-byte rows) that rows of 32-bit words are widened to
inline int64_t w32_row_words(int64_t K) { return (bmx::words_for(K) + 1) / 2 * 2; }

struct QuantWs {
  size_t planes_off, wb_off, rowsum_off, wrowsum_off, tmp_off, total;
};

// bits_w = 1: sign-packed weights [N][Kw].  bits_w > 1: weight planes [N * bits_w][padded K]
// like the activations', their (unused) row sums, and the int32 results per weight plane.
QuantWs quant_ws(int64_t M, int64_t N, int64_t K, int bits_a, int bits_w) {
  const int64_t Kw = bmx::words_for(K);
  QuantWs q;
  q.planes_off = 0;
  q.wb_off = round256((size_t)bits_a * M * bmx::padded_words(K) * 8);
  q.rowsum_off = q.wb_off + round256(bits_w == 1 ? (size_t)N * Kw * 8
                                                   : (size_t)bits_w * N * bmx::padded_words(K) * 8);
  q.wrowsum_off = q.rowsum_off + round256((size_t)M * 4);
  q.tmp_off = q.wrowsum_off + (bits_w == 1 ? 0 : round256((size_t)N * 4));
  q.total = q.tmp_off + (bits_w == 1 ? 0 : round256((size_t)M * N * bits_w * 4));
  return q;
}

}  // namespace

namespace bmx {
static thread_local char last_kernel_name[160] = "";
void note_kernel(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(last_kernel_name, sizeof(last_kernel_name), fmt, ap);
  va_end(ap);
}
extern int conv_filters_per_wave, conv_path;
extern int gemm_tune_rows, gemm_tune_ksplit, gemm_tune_order;
}

extern "C" {

// Kernel-selection hook (keys documented at its declaration).
int bmx_tune_set(int key, int value) {
  if (key == 0) {  // everything back to the automatic choice
    bmx::conv_filters_per_wave = bmx::gemm_tune_rows = bmx::gemm_tune_ksplit = bmx::gemm_tune_order = 0;
    bmx::conv_path = bmx::gemm_engine = bmx::gemm_mfma_ksplit = bmx::gemm_mfma_tile = bmx::gemm_fp4_split = bmx::gemm_fp4_half = bmx::gemm_fp4_band = bmx::gemm_fp4_tall = bmx::conv_ws_x4 = bmx::fc_small = 0;
    return BMX_OK;
  }
  if (key == 1) bmx::conv_filters_per_wave = value;
  else if (key == 2) bmx::gemm_tune_rows = value;
  else if (key == 3) bmx::gemm_tune_ksplit = value;
  else if (key == 4) bmx::gemm_tune_order = value;
  else if (key == 5) bmx::conv_path = value;
  else if (key == 7) bmx::gemm_engine = value;
  else if (key == 8) bmx::gemm_mfma_ksplit = value;
  else if (key == 9) bmx::gemm_mfma_tile = value;
  else if (key == 10) bmx::gemm_fp4_split = value;
  else if (key == 11) bmx::gemm_fp4_half = value;
  else if (key == 12) bmx::gemm_fp4_band = value;
  else if (key == 13) bmx::gemm_fp4_tall = value;
  else if (key == 14) bmx::conv_ws_x4 = value;
  else if (key == 15) bmx::fc_small = value;
  else return BMX_ERR_UNSUPPORTED;
  return BMX_OK;
}

int bmx_version(void) { return 200; }

const char* bmx_last_kernel(void) { return bmx::last_kernel_name; }

int bmx_probe_valu(int workgroups, int iters, unsigned long long* out3, int* wall_clock_khz, void* stream) {
  if (workgroups <= 0 || iters <= 0 || workgroups > (1 << 20) || iters > (1 << 24)) return BMX_ERR_SHAPE;
  if (!out3 || !wall_clock_khz) return BMX_ERR_NULL;
  if (misaligned(out3, 8)) return BMX_ERR_ALIGN;
  int dev = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess)
    return BMX_ERR_HIP;
  *wall_clock_khz = khz;
  return hip_status(bmx::launch_probe_valu(workgroups, iters, out3, (hipStream_t)stream));
}

const char* bmx_status_string(int status) {
  switch (status) {
    case BMX_OK: return "BMX_OK";
    case BMX_ERR_NULL: return "BMX_ERR_NULL: required pointer is NULL";
    case BMX_ERR_SHAPE: return "BMX_ERR_SHAPE: invalid size";
    case BMX_ERR_LD: return "BMX_ERR_LD: leading dimension too small";
    case BMX_ERR_ALIGN: return "BMX_ERR_ALIGN: misaligned pointer";
    case BMX_ERR_UNSUPPORTED: return "BMX_ERR_UNSUPPORTED: argument outside the supported set";
    case BMX_ERR_WORKSPACE: return "BMX_ERR_WORKSPACE: workspace missing or too small";
    case BMX_ERR_HIP: return "BMX_ERR_HIP: HIP runtime error";
    default: return "unknown status";
  }
}

size_t bmx_workspace_bytes(int op, const int64_t* dims, int ndims) {
  if (!dims) return 0;
  switch (op) {
    case BMX_OP_BINARY_FC: {
      if (ndims != 3 || dims[0] < 0 || dims[1] <= 0 || dims[1] >= kMaxK || dims[2] < 0) return 0;
      return round256((size_t)(dims[0] > 0 ? dims[0] : 1) * bmx::padded_words(dims[1]) * 8);
    }
    case BMX_OP_BINARY_CONV2D: {
      if (ndims != 9) return 0;
      ConvGeom g;
      if (conv_check((int)dims[0], (int)dims[1], (int)dims[2], (int)dims[3], (int)dims[4],
                     (int)dims[5], (int)dims[6], (int)dims[7], (int)dims[8], &g) != BMX_OK)
        return 0;
      const size_t n = dims[0] > 0 ? (size_t)dims[0] : 1;
      return round256(n * (dims[2] + 2 * dims[8]) * (dims[3] + 2 * dims[8]) * g.Cw * 8);
    }
    case BMX_OP_BINARY_CONV2D_BITS: {
      if (ndims != 10 || dims[9] < 0 || dims[9] > 6) return 0;
      ConvGeom g;
      if (conv_check((int)dims[0], (int)dims[1], (int)dims[2], (int)dims[3], (int)dims[4],
                     (int)dims[5], (int)dims[6], (int)dims[7], (int)dims[8], &g) != BMX_OK)
        return 0;
      if (bmx::conv_mfma_ws_takes((int)dims[0], (int)dims[1], (int)dims[2], (int)dims[3], (int)dims[4],
                                  (int)dims[5], (int)dims[6], (int)dims[7], (int)dims[8], (int)dims[9]))
        return 0;  // the convolution kernel writes the bits itself
      const size_t n = dims[0] > 0 ? (size_t)dims[0] : 1;
      return round256(n * (dims[4] > 0 ? dims[4] : 1) * g.Ho * g.Wo * 4);
    }
    case BMX_OP_XNOR_GEMM_W32: {
      if (ndims != 3 || dims[0] < 0 || dims[1] < 0 || dims[2] <= 0 || dims[2] >= kMaxK) return 0;
      const int64_t ld = w32_row_words(dims[2]);
      return round256((size_t)(dims[0] > 0 ? dims[0] : 1) * ld * 8) +
             round256((size_t)(dims[1] > 0 ? dims[1] : 1) * ld * 8);
    }
    case BMX_OP_QUANT_GEMM: {
      if (ndims != 5 || dims[0] < 0 || dims[1] < 0 || dims[2] <= 0 || dims[2] >= kMaxK) return 0;
      if (dims[3] < 1 || dims[3] > 8 || dims[4] < 1 || dims[4] > 8) return 0;
      return quant_ws(dims[0] > 0 ? dims[0] : 1, dims[1] > 0 ? dims[1] : 1, dims[2], (int)dims[3],
                      (int)dims[4])
          .total;
    }
    default: return 0;
  }
}

int bmx_binarize_pack(const float* x, int64_t rows, int64_t cols, int64_t ldx, int pack_dim,
                      uint64_t* out, int64_t out_ld_words, void* stream) {
  if (pack_dim != 0 && pack_dim != 1) return BMX_ERR_UNSUPPORTED;
  if (rows < 0 || cols < 0) return BMX_ERR_SHAPE;
  const int64_t R = pack_dim ? rows : cols;
  const int64_t K = pack_dim ? cols : rows;
  if (R == 0) return BMX_OK;
  if (K <= 0 || K >= kMaxK) return BMX_ERR_SHAPE;
  if (!x || !out) return BMX_ERR_NULL;
  if (ldx < cols) return BMX_ERR_LD;
  if (out_ld_words < bmx::words_for(K)) return BMX_ERR_LD;
  if (misaligned(x, 4) || misaligned(out, 8)) return BMX_ERR_ALIGN;
  hipStream_t s = (hipStream_t)stream;
  if (pack_dim)
    return hip_status(bmx::launch_pack_rows(x, rows, cols, ldx, out, out_ld_words, s));
  return hip_status(bmx::launch_pack_strided(x, 1, rows, cols, ldx, 0, out, out_ld_words, s));
}

int bmx_unpack_pm1(const uint64_t* bits, int64_t rows, int64_t K, int64_t ld_words, float* out,
                   int64_t ldo, void* stream) {
  if (rows < 0) return BMX_ERR_SHAPE;
  if (K <= 0 || K >= kMaxK) return BMX_ERR_SHAPE;
  if (rows == 0) return BMX_OK;
  if (!bits || !out) return BMX_ERR_NULL;
  if (ld_words < bmx::words_for(K) || ldo < K) return BMX_ERR_LD;
  if (misaligned(bits, 8) || misaligned(out, 4)) return BMX_ERR_ALIGN;
  return hip_status(bmx::launch_unpack_pm1(bits, rows, K, ld_words, out, ldo, (hipStream_t)stream));
}

namespace {
int xnor_gemm_checked(const uint64_t* A, int64_t lda_w, const uint64_t* B, int64_t ldb_w, int32_t* C,
                      int64_t ldc, int M, int N, int K, void* stream, bool as_count) {
  if (M < 0 || N < 0) return BMX_ERR_SHAPE;
  if (K <= 0 || K >= kMaxK) return BMX_ERR_SHAPE;
  if (M == 0 || N == 0) return BMX_OK;
  if (!A || !B || !C) return BMX_ERR_NULL;
  const int64_t Kw = bmx::words_for(K);
  if (lda_w < Kw || ldb_w < Kw || ldc < N) return BMX_ERR_LD;
  if (misaligned(A, 8) || misaligned(B, 8) || misaligned(C, 4)) return BMX_ERR_ALIGN;
  return hip_status(bmx::launch_xnor_gemm((const uint32_t*)A, false, lda_w * 2, B, ldb_w, M, N, K,
                                          nullptr, C, nullptr, nullptr, nullptr, ldc, (hipStream_t)stream,
                                          as_count));
}
}  // namespace

int bmx_xnor_gemm(const uint64_t* A, int64_t lda_w, const uint64_t* B, int64_t ldb_w, int32_t* C,
                  int64_t ldc, int M, int N, int K, void* stream) {
  return xnor_gemm_checked(A, lda_w, B, ldb_w, C, ldc, M, N, K, stream, false);
}

int bmx_xnor_gemm_count(const uint64_t* A, int64_t lda_w, const uint64_t* B, int64_t ldb_w, int32_t* C,
                        int64_t ldc, int M, int N, int K, void* stream) {
  return xnor_gemm_checked(A, lda_w, B, ldb_w, C, ldc, M, N, K, stream, true);
}

int bmx_widen_words32(const uint32_t* in, int64_t rows, int64_t K, int64_t ld_dwords, uint64_t* out,
                      int64_t out_ld_words, void* stream) {
  if (rows < 0) return BMX_ERR_SHAPE;
  if (K <= 0 || K >= kMaxK) return BMX_ERR_SHAPE;
  if (rows == 0) return BMX_OK;
  if (rows * bmx::words_for(K) >= ((int64_t)1 << 38)) return BMX_ERR_SHAPE;
  if (!in || !out) return BMX_ERR_NULL;
  if (ld_dwords < (K + 31) / 32 || out_ld_words < bmx::words_for(K)) return BMX_ERR_LD;
  if (misaligned(in, 4) || misaligned(out, 8)) return BMX_ERR_ALIGN;
  return hip_status(bmx::launch_widen_words32(in, rows, K, ld_dwords, out, out_ld_words, (hipStream_t)stream));
}

int bmx_xnor_gemm_w32(const uint32_t* A, int64_t lda_dw, const uint32_t* B, int64_t ldb_dw, int32_t* C,
                      int64_t ldc, int M, int N, int K, void* workspace, size_t workspace_bytes,
                      void* stream) {
  if (M < 0 || N < 0) return BMX_ERR_SHAPE;
  if (K <= 0 || K >= kMaxK) return BMX_ERR_SHAPE;
  if (M == 0 || N == 0) return BMX_OK;
  if (!A || !B || !C) return BMX_ERR_NULL;
  const int64_t Kd = ((int64_t)K + 31) / 32;
  if (lda_dw < Kd || ldb_dw < Kd || ldc < N) return BMX_ERR_LD;
  if (misaligned(A, 4) || misaligned(B, 4) || misaligned(C, 4)) return BMX_ERR_ALIGN;
  // An operand whose rows are whole, 8-byte aligned 64-bit words already IS the 64-bit layout
  // (same bytes); any other (odd dword count or stride, 4-byte aligned base) is widened first.
  auto direct = [&](const uint32_t* X, int64_t ld) { return !misaligned(X, 8) && (ld & 1) == 0 && (Kd & 1) == 0; };
  const bool da = direct(A, lda_dw), db = direct(B, ldb_dw);
  const int64_t ldw = w32_row_words(K);
  const size_t a_bytes = round256((size_t)M * ldw * 8), b_bytes = round256((size_t)N * ldw * 8);
  const uint64_t *A64 = (const uint64_t*)A, *B64 = (const uint64_t*)B;
  int64_t lda_w = lda_dw / 2, ldb_w = ldb_dw / 2;
  hipStream_t s = (hipStream_t)stream;
  if (!da || !db) {
    if (!workspace || workspace_bytes < a_bytes + b_bytes) return BMX_ERR_WORKSPACE;
    if (misaligned(workspace, 16)) return BMX_ERR_ALIGN;
  }
  if (!da) {
    uint64_t* wa = (uint64_t*)workspace;
    if (bmx::launch_widen_words32(A, M, K, lda_dw, wa, ldw, s) != hipSuccess) return BMX_ERR_HIP;
    A64 = wa;
    lda_w = ldw;
  }
  if (!db) {
    uint64_t* wb = (uint64_t*)((char*)workspace + a_bytes);
    if (bmx::launch_widen_words32(B, N, K, ldb_dw, wb, ldw, s) != hipSuccess) return BMX_ERR_HIP;
    B64 = wb;
    ldb_w = ldw;
  }
  return xnor_gemm_checked(A64, lda_w, B64, ldb_w, C, ldc, M, N, K, stream, false);
}

namespace {
// Argument checks shared by the two fully connected entry points (zero-sized problems pass).
int fc_check(const float* x, int64_t ldx, const uint64_t* Wp, int64_t ldw_w, const float* alpha, int batch,
             int in_features, int out_features, int32_t* out_i32, float* out_f32, int64_t ldo) {
  if (batch < 0 || out_features < 0) return BMX_ERR_SHAPE;
  if (in_features <= 0 || in_features >= kMaxK) return BMX_ERR_SHAPE;
  if (batch == 0 || out_features == 0) return BMX_OK;
  if (!x || !Wp) return BMX_ERR_NULL;
  if ((out_i32 == nullptr) == (out_f32 == nullptr)) return BMX_ERR_NULL;
  if (out_i32 && alpha) return BMX_ERR_UNSUPPORTED;
  const int64_t Kw = bmx::words_for(in_features);
  if (ldx < in_features || ldw_w < Kw || ldo < out_features) return BMX_ERR_LD;
  if (misaligned(x, 4) || misaligned(Wp, 8) || misaligned(alpha, 4) || misaligned(out_i32, 4) ||
      misaligned(out_f32, 4))
    return BMX_ERR_ALIGN;
  return BMX_OK;
}

// Pack the activations into chunk-padded rows at xp (the scalar side of the GEMM kernel reads
// whole chunks), then the GEMM with the epilogue.
int fc_launch(const float* x, int64_t ldx, const uint64_t* Wp, int64_t ldw_w, const float* alpha, int batch,
              int in_features, int out_features, int32_t* out_i32, float* out_f32, int64_t ldo, uint64_t* xp,
              hipStream_t s) {
  hipError_t small = hipSuccess;  // a layer of a few microseconds or less: one launch, no workspace
  if (bmx::launch_fc_small(x, ldx, Wp, ldw_w, alpha, batch, in_features, out_features, out_i32, out_f32, ldo, s, &small))
    return hip_status(small);
  const int64_t ldp = bmx::padded_words(in_features);
  hipError_t e = bmx::launch_pack_rows_padded(x, batch, in_features, ldx, xp, ldp, s);
  if (e != hipSuccess) return BMX_ERR_HIP;
  return hip_status(bmx::launch_xnor_gemm((const uint32_t*)xp, true, ldp * 2, Wp, ldw_w, batch,
                                          out_features, in_features, alpha, out_i32, out_f32,
                                          nullptr, nullptr, ldo, s));
}
}  // namespace

int bmx_binary_fc(const float* x, int64_t ldx, const uint64_t* Wp, int64_t ldw_w,
                  const float* alpha, int batch, int in_features, int out_features,
                  int32_t* out_i32, float* out_f32, int64_t ldo, void* workspace,
                  size_t workspace_bytes, void* stream) {
  const int rc = fc_check(x, ldx, Wp, ldw_w, alpha, batch, in_features, out_features, out_i32, out_f32, ldo);
  if (rc != BMX_OK) return rc;
  if (batch == 0 || out_features == 0) return BMX_OK;
  const int64_t dims[3] = {batch, in_features, out_features};
  const size_t need = bmx_workspace_bytes(BMX_OP_BINARY_FC, dims, 3);
  if (!workspace || workspace_bytes < need) return BMX_ERR_WORKSPACE;
  if (misaligned(workspace, 16)) return BMX_ERR_ALIGN;
  return fc_launch(x, ldx, Wp, ldw_w, alpha, batch, in_features, out_features, out_i32, out_f32, ldo,
                   (uint64_t*)workspace, (hipStream_t)stream);
}

int bmx_binary_fc_static(const float* x, int64_t ldx, const uint64_t* Wp, int64_t ldw_w,
                         const float* alpha, int batch, int in_features, int out_features,
                         int32_t* out_i32, float* out_f32, int64_t ldo, void* stream) {
  const int rc = fc_check(x, ldx, Wp, ldw_w, alpha, batch, in_features, out_features, out_i32, out_f32, ldo);
  if (rc != BMX_OK) return rc;
  if (batch == 0 || out_features == 0) return BMX_OK;
  const int64_t dims[3] = {batch, in_features, out_features};
  if (bmx_workspace_bytes(BMX_OP_BINARY_FC, dims, 3) > (size_t)BMX_STATIC_SCRATCH_BYTES)
    return BMX_ERR_WORKSPACE;  // the packed activations do not fit the library's own scratch
  // The address of this GPU's copy of the array, asked for once per device (with that device
  // current) and kept: every GPU holds its own copy at its own address.
  static std::mutex mu;
  static void* resolved[64];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return BMX_ERR_HIP;
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (!resolved[dev]) {
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return BMX_ERR_HIP;
      resolved[dev] = p;
    }
    ptr = resolved[dev];
  }
  // (the pack kernel writes every word of every padded row it hands to the GEMM, so nothing of
  // a previous call's contents is ever read and nothing needs clearing)
  return fc_launch(x, ldx, Wp, ldw_w, alpha, batch, in_features, out_features, out_i32, out_f32, ldo,
                   (uint64_t*)ptr, (hipStream_t)stream);
}

int bmx_binary_fc_packed(const uint64_t* xp, int64_t ldx_w, const uint64_t* Wp, int64_t ldw_w,
                         const float* alpha, int batch, int in_features, int out_features,
                         int32_t* out_i32, float* out_f32, uint64_t* out_bits, const float* thr,
                         int64_t ldo, void* stream) {
  if (batch < 0 || out_features < 0) return BMX_ERR_SHAPE;
  if (in_features <= 0 || in_features >= kMaxK) return BMX_ERR_SHAPE;
  if (batch == 0 || out_features == 0) return BMX_OK;
  if (!xp || !Wp) return BMX_ERR_NULL;
  if ((out_i32 != nullptr) + (out_f32 != nullptr) + (out_bits != nullptr) != 1) return BMX_ERR_NULL;
  if (out_i32 && alpha) return BMX_ERR_UNSUPPORTED;
  if (thr && !out_bits) return BMX_ERR_UNSUPPORTED;
  const int64_t Kw = bmx::words_for(in_features);
  if (ldx_w < Kw || ldw_w < Kw) return BMX_ERR_LD;
  if (ldo < (out_bits ? bmx::words_for(out_features) : (int64_t)out_features)) return BMX_ERR_LD;
  if (misaligned(xp, 8) || misaligned(Wp, 8) || misaligned(alpha, 4) || misaligned(out_i32, 4) ||
      misaligned(out_f32, 4) || misaligned(out_bits, 8) || misaligned(thr, 4))
    return BMX_ERR_ALIGN;
  return hip_status(bmx::launch_xnor_gemm((const uint32_t*)xp, false, ldx_w * 2, Wp, ldw_w, batch,
                                          out_features, in_features, alpha, out_i32, out_f32,
                                          out_bits, thr, ldo, (hipStream_t)stream));
}

int64_t bmx_conv_weight_row_words(int C, int KH, int KW) {
  ConvGeom g;
  if (conv_check(1, C, KH, KW, 1, KH, KW, 1, 0, &g) != BMX_OK) return 0;
  return bmx::conv_weight_row_words((int64_t)KH * KW * g.Cw);
}

int bmx_pack_conv_weights(const float* w_oihw, int O, int C, int KH, int KW, uint64_t* Wp,
                          void* stream) {
  ConvGeom g;
  // geometry rules for the kernel window only; image size does not matter here
  const int rc = conv_check(1, C, KH, KW, O, KH, KW, 1, 0, &g);
  if (rc != BMX_OK) return rc;
  if (O == 0) return BMX_OK;
  if (!w_oihw || !Wp) return BMX_ERR_NULL;
  if (misaligned(w_oihw, 4) || misaligned(Wp, 8)) return BMX_ERR_ALIGN;
  return hip_status(bmx::launch_pack_conv_weights(w_oihw, O, C, KH, KW, Wp, (hipStream_t)stream));
}

int bmx_pack_nchw(const float* x, int N, int C, int H, int W, int pad, uint64_t* xp, void* stream) {
  if (N < 0 || C <= 0 || H <= 0 || W <= 0) return BMX_ERR_SHAPE;
  if (pad < 0 || pad > 6) return BMX_ERR_UNSUPPORTED;
  if (N > 65535 || (int64_t)(H + 2 * pad) * (W + 2 * pad) >= ((int64_t)1 << 31) ||
      bmx::words_for(C) > 65535)
    return BMX_ERR_SHAPE;
  if (N == 0) return BMX_OK;
  if (!x || !xp) return BMX_ERR_NULL;
  if (misaligned(x, 4) || misaligned(xp, 8)) return BMX_ERR_ALIGN;
  return hip_status(bmx::launch_pack_nchw(x, N, C, H, W, pad, xp, (hipStream_t)stream));
}

int bmx_binary_conv2d_packed(const uint64_t* xp, int N, int C, int H, int W, const uint64_t* Wp,
                             int O, int KH, int KW, int stride, int pad, const float* alpha,
                             int32_t* out_i32, float* out_f32, void* stream) {
  ConvGeom g;
  const int rc = conv_check(N, C, H, W, O, KH, KW, stride, pad, &g);
  if (rc != BMX_OK) return rc;
  if (N == 0 || O == 0) return BMX_OK;
  if (!xp || !Wp) return BMX_ERR_NULL;
  if ((out_i32 == nullptr) == (out_f32 == nullptr)) return BMX_ERR_NULL;
  if (out_i32 && alpha) return BMX_ERR_UNSUPPORTED;
  if (misaligned(xp, 8) || misaligned(Wp, 8) || misaligned(alpha, 4) || misaligned(out_i32, 4) ||
      misaligned(out_f32, 4))
    return BMX_ERR_ALIGN;
  return hip_status(bmx::launch_binary_conv2d(xp, N, C, H, W, Wp, O, KH, KW, stride, pad, alpha,
                                              out_i32, out_f32, (hipStream_t)stream));
}

int bmx_binary_conv2d_bits(const uint64_t* xp, int N, int C, int H, int W, const uint64_t* Wp, int O,
                           int KH, int KW, int stride, int pad, const float* alpha, const float* thr,
                           uint64_t* out_xp, int out_pad, void* workspace, size_t workspace_bytes,
                           void* stream) {
  ConvGeom g;
  const int rc = conv_check(N, C, H, W, O, KH, KW, stride, pad, &g);
  if (rc != BMX_OK) return rc;
  if (out_pad < 0 || out_pad > 6) return BMX_ERR_UNSUPPORTED;
  if (N > 65535 || bmx::words_for(O) > 65535 ||
      (int64_t)(g.Ho + 2 * out_pad) * (g.Wo + 2 * out_pad) >= ((int64_t)1 << 31))
    return BMX_ERR_SHAPE;
  if (N == 0 || O == 0) return BMX_OK;  // an image of zero channels has no words
  if (!xp || !Wp || !out_xp) return BMX_ERR_NULL;
  if (misaligned(xp, 8) || misaligned(Wp, 8) || misaligned(alpha, 4) || misaligned(thr, 4) ||
      misaligned(out_xp, 8))
    return BMX_ERR_ALIGN;
  // where the size query answered 0 the kernel that writes the bits itself must run, and it
  // reads filter rows in 16-byte pieces
  if (bmx::conv_mfma_ws_takes(N, C, H, W, O, KH, KW, stride, pad, out_pad) && misaligned(Wp, 16))
    return BMX_ERR_ALIGN;
  hipStream_t s = (hipStream_t)stream;
  hipError_t err = hipSuccess;
  if (bmx::launch_conv_mfma_ws(xp, N, C, H, W, Wp, O, KH, KW, stride, pad, alpha, nullptr, nullptr, out_xp, thr,
                               out_pad, s, &err))
    return hip_status(err);
  // every other shape: the fp32 result through the workspace, then the channel pack with the
  // same compare
  const size_t need = round256((size_t)N * O * g.Ho * g.Wo * 4);
  if (!workspace || workspace_bytes < need) return BMX_ERR_WORKSPACE;
  if (misaligned(workspace, 16)) return BMX_ERR_ALIGN;
  float* tmp = (float*)workspace;
  err = bmx::launch_binary_conv2d(xp, N, C, H, W, Wp, O, KH, KW, stride, pad, alpha, nullptr, tmp, s);
  if (err != hipSuccess) return BMX_ERR_HIP;
  return hip_status(bmx::launch_pack_nchw_thr(tmp, N, O, g.Ho, g.Wo, out_pad, thr, out_xp, s));
}

int bmx_binary_conv2d(const float* x, int N, int C, int H, int W, const uint64_t* Wp, int O,
                      int KH, int KW, int stride, int pad, const float* alpha, int32_t* out_i32,
                      float* out_f32, void* workspace, size_t workspace_bytes, void* stream) {
  ConvGeom g;
  const int rc = conv_check(N, C, H, W, O, KH, KW, stride, pad, &g);
  if (rc != BMX_OK) return rc;
  if (N == 0 || O == 0) return BMX_OK;
  if (!x || !Wp) return BMX_ERR_NULL;
  if ((out_i32 == nullptr) == (out_f32 == nullptr)) return BMX_ERR_NULL;
  if (out_i32 && alpha) return BMX_ERR_UNSUPPORTED;
  if (misaligned(x, 4) || misaligned(Wp, 8) || misaligned(alpha, 4) || misaligned(out_i32, 4) ||
      misaligned(out_f32, 4))
    return BMX_ERR_ALIGN;
  const int64_t dims[9] = {N, C, H, W, O, KH, KW, stride, pad};
  const size_t need = bmx_workspace_bytes(BMX_OP_BINARY_CONV2D, dims, 9);
  if (!workspace || workspace_bytes < need) return BMX_ERR_WORKSPACE;
  if (misaligned(workspace, 16)) return BMX_ERR_ALIGN;
  uint64_t* xp = (uint64_t*)workspace;
  int st = bmx_pack_nchw(x, N, C, H, W, pad, xp, stream);
  if (st != BMX_OK) return st;
  return bmx_binary_conv2d_packed(xp, N, C, H, W, Wp, O, KH, KW, stride, pad, alpha, out_i32,
                                  out_f32, stream);
}

int bmx_quant_gemm(const float* a, int64_t lda, int bits_a, const float* w, int64_t ldw,
                   int bits_w, int M, int N, int K, int32_t* out_i32_scaled, float* out_f32,
                   int64_t ldo, void* workspace, size_t workspace_bytes, void* stream) {
  if (M < 0 || N < 0) return BMX_ERR_SHAPE;
  if (K <= 0 || K >= kMaxK) return BMX_ERR_SHAPE;
  if (bits_a < 1 || bits_a > 8 || bits_w < 1 || bits_w > 8) return BMX_ERR_UNSUPPORTED;
  if ((int64_t)K * ((1 << bits_a) - 1) * ((1 << bits_w) - 1) >= ((int64_t)1 << 31)) return BMX_ERR_SHAPE;
  if ((int64_t)M * bits_a >= ((int64_t)1 << 31) || (int64_t)N * bits_w >= ((int64_t)1 << 31))
    return BMX_ERR_SHAPE;
  if (M == 0 || N == 0) return BMX_OK;
  if (!a || !w) return BMX_ERR_NULL;
  if (!out_i32_scaled && !out_f32) return BMX_ERR_NULL;
  if (lda < K || ldw < K || ldo < N) return BMX_ERR_LD;
  if (misaligned(a, 4) || misaligned(w, 4) || misaligned(out_i32_scaled, 4) ||
      misaligned(out_f32, 4))
    return BMX_ERR_ALIGN;
  const QuantWs q = quant_ws(M, N, K, bits_a, bits_w);
  if (!workspace || workspace_bytes < q.total) return BMX_ERR_WORKSPACE;
  if (misaligned(workspace, 16)) return BMX_ERR_ALIGN;
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  uint64_t* planes = (uint64_t*)(ws + q.planes_off);
  uint64_t* wb = (uint64_t*)(ws + q.wb_off);
  int32_t* rowsum = (int32_t*)(ws + q.rowsum_off);
  const int64_t Kw = bmx::words_for(K);
  const int64_t ldp = bmx::padded_words(K);
  if (bits_w > 1) {
    // k-bit weights: quantise both operands into bit planes, run the 1-bit-weight form against
    // every weight plane (they are N * bits_w columns of one GEMM), add the planes up weighted
    // by their powers of two: sum_r 2^r (2 sum_p 2^p pc(A_p & W_r) - rowsum) = S
    uint64_t* wplanes = wb;
    int32_t* wrowsum = (int32_t*)(ws + q.wrowsum_off);
    int32_t* tmp = (int32_t*)(ws + q.tmp_off);
    hipError_t e = bmx::launch_quant_pack(a, M, K, lda, bits_a, planes, ldp, rowsum, nullptr, 0, 0, nullptr, 0, s);
    if (e != hipSuccess) return BMX_ERR_HIP;
    e = bmx::launch_quant_pack(w, N, K, ldw, bits_w, wplanes, ldp, wrowsum, nullptr, 0, 0, nullptr, 0, s, true);
    if (e != hipSuccess) return BMX_ERR_HIP;
    e = bmx::launch_plane_gemm((const uint32_t*)planes, ldp * 2, bits_a, rowsum, wplanes, ldp, M, N * bits_w, K,
                               tmp, nullptr, (int64_t)N * bits_w, s);
    if (e != hipSuccess) return BMX_ERR_HIP;
    const float denom = (float)(((1 << bits_a) - 1) * ((1 << bits_w) - 1));
    return hip_status(bmx::launch_quant_combine(tmp, M, N, bits_w, denom, out_i32_scaled, out_f32, ldo, s));
  }
  // one launch quantises + plane-packs the activations and sign-packs the weights
  hipError_t e = bmx::launch_quant_pack(a, M, K, lda, bits_a, planes, ldp, rowsum, w, N, ldw, wb, Kw, s);
  if (e != hipSuccess) return BMX_ERR_HIP;
  return hip_status(bmx::launch_plane_gemm((const uint32_t*)planes, ldp * 2, bits_a, rowsum, wb, Kw,
                                           M, N, K, out_i32_scaled, out_f32, ldo, s));
}

int bmx_alpha_mean_abs(const float* w, int64_t rows, int64_t cols, int64_t ldw, float* alpha,
                       void* stream) {
  if (rows < 0) return BMX_ERR_SHAPE;
  if (cols <= 0) return BMX_ERR_SHAPE;
  if (rows == 0) return BMX_OK;
  if (!w || !alpha) return BMX_ERR_NULL;
  if (ldw < cols) return BMX_ERR_LD;
  if (misaligned(w, 4) || misaligned(alpha, 4)) return BMX_ERR_ALIGN;
  return hip_status(bmx::launch_alpha_mean_abs(w, rows, cols, ldw, alpha, (hipStream_t)stream));
}

}  // extern "C"
