/* bmx.h - C ABI of the MI355X (gfx950) binary-layer library.
 *
 * The library computes the inference hot path of the binary layers of BMXNet
 * (arXiv 1705.09864): sign-binarise and bit-pack fp32 activations and weights
 * (paper Sec. 1, Sec. 2.2.1), then evaluate fully connected and convolution
 * layers as xor + popcount dot products (Sec. 2.2.1; conv-as-GEMM mapping of
 * Sec. 3.1), plus a k-bit generalisation built on the Eq. 1 quantiser.
 *
 * Conventions common to every call
 *   - Returns an int status: BMX_OK (0) or a negative BMX_ERR_* code.  Nothing
 *     throws or aborts.  All argument checks run on the host before any launch;
 *     on an error return no kernel was launched and no output was touched.
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates nothing.  Scratch memory is passed in by the caller (`workspace`,
 *     sized with bmx_workspace_bytes); the one exception, bmx_binary_fc_static,
 *     says so at its declaration.
 *   - Results never depend on earlier calls.  The library does hold process-wide
 *     state of two kinds, neither of which changes a result: the kernel-selection
 *     settings of bmx_tune_set (a measurement and test hook, see there) and
 *     per-device addresses looked up once (bmx_binary_fc_static).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     are asynchronous on it; the caller synchronises.
 *   - Inputs and outputs must not overlap.
 *   - Zero-sized problems (a row/batch/column count of 0) return BMX_OK without
 *     launching.  Negative counts and K <= 0 give BMX_ERR_SHAPE.
 *   - K (the dot-product length) must be < 2^24 so that float(dot) is exact.
 *
 * Packed format (part of the ABI; Sec. 2.2.1 BINARY_WORD, 64-bit flavour)
 *   uint64 little-endian words; element k of a row is bit (k mod 64) of word
 *   floor(k / 64), least significant bit first; bit 1 <-> +1, bit 0 <-> -1 with
 *   sign(0) = +1, i.e. bit = (x >= 0.0f) (IEEE compare: -0.0 -> 1, NaN -> 0);
 *   unused tail bits of the last word are 0.  Row stride ld_words >=
 *   ceil(K / 64); words beyond ceil(K / 64) in a row are neither read nor
 *   written.  Packed pointers must be 8-byte aligned.
 *
 * Output form
 *   The integer result of a binary dot product is the +-1 dot product
 *       dot = K - 2 * popcount(a XOR w),
 *   which equals the float layer restricted to -1/+1 (Sec. 2.2.2).  The xnor
 *   count of the paper's listing is (dot + K) / 2 (Eq. 2).
 */
#ifndef BMX_H
#define BMX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BMX_OK 0
#define BMX_ERR_NULL (-1)        /* a required pointer is NULL */
#define BMX_ERR_SHAPE (-2)       /* negative size, K <= 0, K >= 2^24, empty conv output, or more
                                    than 2^31 - 1 output pixels / 65535 images / 262140 filters */
#define BMX_ERR_LD (-3)          /* a leading dimension is smaller than the row it must hold */
#define BMX_ERR_ALIGN (-4)       /* pointer not aligned (packed: 8 bytes, fp32/int32: 4 bytes) */
#define BMX_ERR_UNSUPPORTED (-5) /* pack_dim, kernel size, stride, bit width outside the contract */
#define BMX_ERR_WORKSPACE (-6)   /* workspace NULL or smaller than bmx_workspace_bytes says */
#define BMX_ERR_HIP (-7)         /* the HIP runtime reported an error at launch */

/* Operation selectors for bmx_workspace_bytes. */
#define BMX_OP_BINARY_FC 1     /* dims = {batch, in_features, out_features} */
#define BMX_OP_BINARY_CONV2D 2 /* dims = {N, C, H, W, O, KH, KW, stride, pad} */
#define BMX_OP_QUANT_GEMM 3    /* dims = {M, N, K, bits_a, bits_w} */
#define BMX_OP_BINARY_CONV2D_BITS 4 /* dims = {N, C, H, W, O, KH, KW, stride, pad, out_pad} */
#define BMX_OP_XNOR_GEMM_W32 5 /* dims = {M, N, K} */

/* Sign-binarise and bit-pack (Sec. 1: binarisation with the sign function, 64
 * values per word; Sec. 3.1: the per-forward-pass input binarisation step).
 *   x        fp32 [rows, cols], row-major, leading dimension ldx >= cols (elements).
 *   pack_dim 1: pack along cols: out is [rows][ceil(cols/64)]  (K contiguous in x);
 *            0: pack along rows: out is [cols][ceil(rows/64)]  (x is stored K x N).
 *   out      uint64, row stride out_ld_words >= ceil(K/64); written in full for the
 *            first ceil(K/64) words of each row (tail bits 0). */
int bmx_binarize_pack(const float* x, int64_t rows, int64_t cols, int64_t ldx, int pack_dim,
                      uint64_t* out, int64_t out_ld_words, void* stream);

/* The inverse of bmx_binarize_pack(pack_dim = 1): out[r][k] = bit k of row r ? +1.0f : -1.0f.
 * A model stored with 1-bit weights (Sec. 2.2.3: the converter's output, 32x smaller than
 * fp32) goes back through this to the +-1 floats every pack routine of the library starts
 * from, e.g. bmx_pack_conv_weights with its private row layout.
 *   bits uint64 [rows, ld_words], ld_words >= ceil(K/64);  out fp32 [rows, ldo], ldo >= K. */
int bmx_unpack_pm1(const uint64_t* bits, int64_t rows, int64_t K, int64_t ld_words, float* out,
                   int64_t ldo, void* stream);

/* xnor GEMM on packed operands (Sec. 2.2.1, the xnor GEMM kernel; output form per
 * Sec. 2.2.2 / Eq. 2):  C[m][n] = K - 2 * sum_i popcount(A[m][i] ^ B[n][i]).
 *   A  uint64 [M, lda_w], B uint64 [N, ldb_w], both packed along K (K contiguous),
 *      tail bits zero.   C  int32 [M, ldc], ldc >= N; overwritten, not accumulated. */
int bmx_xnor_gemm(const uint64_t* A, int64_t lda_w, const uint64_t* B, int64_t ldb_w, int32_t* C,
                  int64_t ldc, int M, int N, int K, void* stream);

/* The same product in the other range of Eq. 2 (Sec. 2.2.2): the xnor count
 *   C[m][n] = number of k with A[m][k] == B[n][k] = (dot + K) / 2, in 0 .. K,
 * which is what the listing of Sec. 2.2.1 accumulates.  Arguments as for bmx_xnor_gemm. */
int bmx_xnor_gemm_count(const uint64_t* A, int64_t lda_w, const uint64_t* B, int64_t ldb_w, int32_t* C,
                        int64_t ldc, int M, int N, int K, void* stream);

/* The 32-bit BINARY_WORD flavour (Sec. 2.2.1: 32 values per word on x86 and ARMv7, 64 on x64).
 * A row of 32-bit words holds element k in bit (k mod 32) of dword floor(k / 32), least
 * significant bit first, unused tail bits 0; rows are ld_dwords >= ceil(K/32) dwords apart and
 * 4-byte aligned.  Little-endian, that is byte for byte the 64-bit row, except that a row may end
 * in (or be strided by) an odd number of dwords and need not start 8-byte aligned.
 * bmx_widen_words32: copy such rows into the library's 64-bit layout (the missing upper half of
 *   a last odd dword becomes 0), for any call that takes packed operands.
 *   in uint32 [rows, ld_dwords];  out uint64 [rows, out_ld_words], out_ld_words >= ceil(K/64).
 * bmx_xnor_gemm_w32: bmx_xnor_gemm on operands of 32-bit words (the xnor_32 kernel of the
 *   paper's Sec. 3.1 evaluation).  An operand whose rows are whole 64-bit words already (even
 *   dword count and stride, 8-byte aligned base) is read in place; any other is widened into
 *   `workspace` first.  workspace >= bmx_workspace_bytes(BMX_OP_XNOR_GEMM_W32, {M, N, K}, 3),
 *   16-byte aligned; it may be NULL when both operands are read in place. */
int bmx_widen_words32(const uint32_t* in, int64_t rows, int64_t K, int64_t ld_dwords, uint64_t* out,
                      int64_t out_ld_words, void* stream);
int bmx_xnor_gemm_w32(const uint32_t* A, int64_t lda_dw, const uint32_t* B, int64_t ldb_dw, int32_t* C,
                      int64_t ldc, int M, int N, int K, void* workspace, size_t workspace_bytes,
                      void* stream);

/* Binary fully connected layer (Sec. 2, QFullyConnected): binarise + pack the fp32
 * activations, xnor GEMM against pre-packed weights, optional scale.
 *   x        fp32 [batch, in_features], leading dimension ldx.
 *   Wp       uint64 [out_features, ldw_w], packed along in_features by
 *            bmx_binarize_pack (pack_dim = 1 on [out, in] weights, or 0 on [in, out]).
 *   alpha    fp32 [out_features] or NULL (= 1).
 *   out_i32 / out_f32   exactly one is non-NULL; both are [batch, ldo], ldo >= out_features.
 *            out_i32 = dot (alpha must be NULL);  out_f32 = alpha[o] * (float)dot.
 *   workspace >= bmx_workspace_bytes(BMX_OP_BINARY_FC, {batch, in, out}, 3), 16-byte aligned. */
int bmx_binary_fc(const float* x, int64_t ldx, const uint64_t* Wp, int64_t ldw_w,
                  const float* alpha, int batch, int in_features, int out_features,
                  int32_t* out_i32, float* out_f32, int64_t ldo, void* workspace,
                  size_t workspace_bytes, void* stream);

/* bmx_binary_fc for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and
 * results as bmx_binary_fc minus the workspace: the packed activations live in a 4 MiB array
 * inside the library's device code (one copy per GPU, held until the process ends).  The call
 * allocates and frees nothing.
 *   - batch * 128 * ceil(in_features / 1024) bytes (the packed, chunk-padded activations, i.e.
 *     bmx_workspace_bytes(BMX_OP_BINARY_FC, ..)) must not exceed 4 MiB: BMX_ERR_WORKSPACE
 *     otherwise, before any launch.
 *   - Every call on one GPU shares that GPU's array: calls that overlap on one GPU (two streams,
 *     two threads) race; calls on one stream are ordered and safe.
 *   - The first call on a device looks the array's address up (hipGetSymbolAddress); make one
 *     call on each device before capturing a graph. */
int bmx_binary_fc_static(const float* x, int64_t ldx, const uint64_t* Wp, int64_t ldw_w,
                         const float* alpha, int batch, int in_features, int out_features,
                         int32_t* out_i32, float* out_f32, int64_t ldo, void* stream);

/* Binary fully connected layer on already packed activations, for chains of binary layers
 * (Sec. 2: QActivation -> QFullyConnected blocks): the layer's result can leave as the packed
 * sign bits the next layer reads, so the fp32 activations between two binary layers are
 * never written or read.
 *   xp       uint64 [batch, ldx_w], packed along in_features (bmx_binarize_pack, or out_bits
 *            of a previous call), tail bits zero.
 *   Wp, alpha as for bmx_binary_fc.
 *   exactly one of out_i32 / out_f32 / out_bits is non-NULL:
 *     out_i32 [batch, ldo] = dot (alpha must be NULL);  out_f32 [batch, ldo] = alpha[o]*(float)dot;
 *     out_bits uint64 [batch, ldo] (ldo in words, >= ceil(out_features/64)): bit o of row b is
 *     (alpha[o] * (float)dot >= thr[o]), the IEEE compare of the fp32 product; with thr NULL
 *     (= 0) exactly what bmx_binarize_pack makes of the out_f32 result (sign(0) = +1); unused
 *     tail bits 0.
 *   thr      fp32 [out_features] or NULL, with out_bits only: the threshold a BatchNorm behind
 *            the layer folds into (see bmx_binary_conv2d_bits). */
int bmx_binary_fc_packed(const uint64_t* xp, int64_t ldx_w, const uint64_t* Wp, int64_t ldw_w,
                         const float* alpha, int batch, int in_features, int out_features,
                         int32_t* out_i32, float* out_f32, uint64_t* out_bits, const float* thr,
                         int64_t ldo, void* stream);

/* Pack OIHW fp32 convolution weights for bmx_binary_conv2d (the offline weight packing
 * of Sec. 2.2.3).  Wp is a matrix of O rows of bmx_conv_weight_row_words(C, KH, KW) words:
 * row o holds filter o, tap (kh, kw) at words (kh*KW + kw)*ceil(C/64) .., word cw of a tap
 * holding channels 64*cw .. 64*cw+63 (missing channels = 0 bits), followed by zero words up
 * to a whole register chunk, and for some K by two words of per-filter constants.  This K
 * order (tap-major, channel-minor), the row length and what lies behind the bits are private
 * to the pair pack/conv; a dot product does not
 * depend on a permutation applied to both operands.
 * bmx_conv_weight_row_words returns the row length in words (0 if KH, KW or C are outside
 * the supported set); the caller allocates O times that many words. */
int64_t bmx_conv_weight_row_words(int C, int KH, int KW);
int bmx_pack_conv_weights(const float* w_oihw, int O, int C, int KH, int KW, uint64_t* Wp,
                          void* stream);

/* Binary 2-D convolution (Sec. 2, QConvolution; Sec. 3.1: M = O, N = batch * Ho * Wo,
 * K = KH * KW * C), NCHW in and out, Ho = (H + 2*pad - KH) / stride + 1 (same for Wo).
 * The fp32 image is treated as zero padded BEFORE the sign function, so a padded tap
 * counts as +1 (sign(0) = +1); this is what makes the layer equal to the float layer on
 * -1/+1 data.  The im2col matrix is never materialised: activations are packed once
 * along C per pixel into `workspace`, taps are gathered by the GEMM kernel.
 *   x      fp32 [N, C, H, W];   Wp from bmx_pack_conv_weights;   alpha fp32 [O] or NULL.
 *   out_i32 / out_f32   exactly one non-NULL, [N, O, Ho, Wo]; out_f32 = alpha[o]*(float)dot.
 *   Supported: KH == KW in {1, 3, 5, 7}, stride in {1, 2}, 0 <= pad < KH, any C >= 1.
 *   workspace >= bmx_workspace_bytes(BMX_OP_BINARY_CONV2D, {N,C,H,W,O,KH,KW,stride,pad}, 9). */
int bmx_binary_conv2d(const float* x, int N, int C, int H, int W, const uint64_t* Wp, int O,
                      int KH, int KW, int stride, int pad, const float* alpha, int32_t* out_i32,
                      float* out_f32, void* workspace, size_t workspace_bytes, void* stream);

/* The two stages of bmx_binary_conv2d as separate calls, for callers that keep the packed
 * image (e.g. to feed several convolutions with the same pad) or time the stages apart.
 * bmx_pack_nchw: the fused im2col + pack step of Sec. 3.1 without the im2col matrix.
 *   xp is [N][H + 2*pad][W + 2*pad][ceil(C/64)] words; pixel (h, w) sits at row h + pad,
 *   column w + pad, and bit c of word cw is (x[n][64*cw + c][h][w] >= 0), missing channels
 *   0 bits.  The halo pixels hold "every real channel = +1" (the sign of the zero padding).
 *   0 <= pad <= 6.
 * bmx_binary_conv2d_packed: the implicit-GEMM stage on an xp packed with the same pad; all
 *   other arguments as for bmx_binary_conv2d (no workspace). */
int bmx_pack_nchw(const float* x, int N, int C, int H, int W, int pad, uint64_t* xp, void* stream);
int bmx_binary_conv2d_packed(const uint64_t* xp, int N, int C, int H, int W, const uint64_t* Wp,
                             int O, int KH, int KW, int stride, int pad, const float* alpha,
                             int32_t* out_i32, float* out_f32, void* stream);

/* Binary convolution whose result leaves as the packed image the next binary convolution
 * reads, for chains of binary blocks (Sec. 2: QActivation -> QConvolution -> BatchNorm, block
 * after block): the fp32 feature map between two binary convolutions is neither written nor
 * read, and the next layer needs no bmx_pack_nchw.
 *   xp, N, C, H, W, Wp, O, KH, KW, stride, pad, alpha as for bmx_binary_conv2d_packed.
 *   thr    fp32 [O] or NULL (= 0): bit o of an output pixel is
 *            (alpha[o] * (float)dot >= thr[o])     (the IEEE compare of the fp32 product),
 *          with thr NULL exactly what bmx_pack_nchw makes of the out_f32 result.  A BatchNorm
 *          behind the convolution folds into thr: gamma * (v - mean) / sigma + beta >= 0 is
 *          v >= mean - beta * sigma / gamma for gamma > 0 (for gamma < 0 negate alpha and thr).
 *   out_xp uint64 [N][Ho + 2*out_pad][Wo + 2*out_pad][ceil(O/64)], the layout of bmx_pack_nchw
 *          for an image of O channels: written whole, the halo with every real channel +1 (the
 *          sign of the next layer's zero padding), missing channels 0 bits.  0 <= out_pad <= 6.
 *   workspace >= bmx_workspace_bytes(BMX_OP_BINARY_CONV2D_BITS, {N,C,H,W,O,KH,KW,stride,pad,
 *          out_pad}, 10): 0 where the convolution kernel writes the bits itself (3 x 3 kernels
 *          over at most 256 channels, 5 x 5 over at most 128, 7 x 7 over at most 64), else room
 *          for the fp32 result, which then passes through the channel pack with the same compare.
 *          For the shapes whose query answers 0, Wp must be 16-byte aligned (BMX_ERR_ALIGN
 *          otherwise): a workspace sized by the query is always enough. */
int bmx_binary_conv2d_bits(const uint64_t* xp, int N, int C, int H, int W, const uint64_t* Wp, int O,
                           int KH, int KW, int stride, int pad, const float* alpha, const float* thr,
                           uint64_t* out_xp, int out_pad, void* workspace, size_t workspace_bytes,
                           void* stream);

/* k-bit activations x 1-bit or k-bit weights (Sec. 1: arbitrary bit widths after DoReFa-Net;
 * Sec. 2.1, Eq. 1).  a in [0, 1] (clamped) is quantised to the integer level
 * q = round((2^bits_a - 1) * a), ties away from zero, and split into bits_a bit planes.
 * bits_w = 1: w is binarised with the sign function.  With wb the weight bits,
 *   S[m][n] = sum_k q[m][k] * sign(w[n][k])
 *           = 2 * sum_p 2^p popcount(plane_p[m] & wb[n]) - sum_p 2^p popcount(plane_p[m]),
 *   out_f32 = (float)S / (float)(2^bits_a - 1)      (the Eq. 1 scale applied once).
 * bits_w in 2..8: w in [-1, 1] (clamped) goes onto [0, 1] by u = (w + 1) / 2, through the same
 * quantiser to the level q_w, and back: w_q = (2 * q_w - L_w) / L_w with L_w = 2^bits_w - 1
 * (Eq. 1 is defined on [0, 1]; the affine pair is DoReFa-Net's).  Then
 *   S[m][n] = sum_k q[m][k] * (2 * q_w[n][k] - L_w),
 *   out_f32 = (float)S / (float)((2^bits_a - 1) * L_w),
 * computed as the bits_w = 1 form against every weight plane, the planes added up by powers
 * of two.  K * (2^bits_a - 1) * (2^bits_w - 1) must stay below 2^31.
 *   a fp32 [M, lda], w fp32 [N, ldw]; out_i32_scaled (S) and out_f32 are [M, ldo]; either
 *   may be NULL, not both.  bits_a, bits_w in 1..8.
 *   workspace >= bmx_workspace_bytes(BMX_OP_QUANT_GEMM, {M, N, K, bits_a, bits_w}, 5). */
int bmx_quant_gemm(const float* a, int64_t lda, int bits_a, const float* w, int64_t ldw,
                   int bits_w, int M, int N, int K, int32_t* out_i32_scaled, float* out_f32,
                   int64_t ldo, void* workspace, size_t workspace_bytes, void* stream);

/* alpha[r] = mean_j |w[r][j]| over cols entries per row (the XNOR-Net weight scale the
 * abstract refers to), accumulated in fp64 and rounded once to fp32.
 *   w fp32 [rows, ldw]; for OIHW conv weights pass rows = O, cols = ldw = C*KH*KW. */
int bmx_alpha_mean_abs(const float* w, int64_t rows, int64_t cols, int64_t ldw, float* alpha,
                       void* stream);

/* Scratch bytes an operation needs (multiple of 256), or 0 if op/dims are invalid. */
size_t bmx_workspace_bytes(int op, const int64_t* dims, int ndims);

/* Kernel-selection hook for measurements and for tests that must reach every kernel
 * variant; not part of the layers the paper defines.  Results never depend on it: every
 * engine and shape computes the same integers (Sec. 2.2.2).  The settings are process-wide
 * state that every later call on any thread sees until they are set back; the hook is not
 * thread safe and must not run concurrently with any other call of the library.  Value 0
 * restores the automatic choice; bmx_tune_set(0, 0) restores it for every key at once.
 * Returns BMX_ERR_UNSUPPORTED for an unknown key.
 *   key 1  filters per wave of the register-stationary convolution kernel; for the short-K
 *          matrix-core kernel, pixel blocks per wave (below 100) or the number of waves the
 *          blocks are dealt out to per filter tile (100 and above)
 *   key 2  rows per wave (8, 16, 32), key 3  K-split waves, key 4  workgroup order of the
 *          xor/popcount GEMM kernel
 *   key 5  convolution kernel: 1 register-stationary, 2 xor/popcount GEMM kernel,
 *          3 one thread per output, 4 matrix cores (GEMM-shaped, 32 x 32 per wave), 5 matrix cores
 *          (short K, filters in LDS), 6 matrix cores (GEMM-shaped, 64 x 64 per wave, operands
 *          staged through LDS)
 *   key 7  GEMM engine: 1 xor/popcount, 2 int8 matrix cores, 3 FP4 matrix cores (kernel chosen by
 *          size), 4 FP4 with 32 x 32 or 64 x 64 per wave and operands through registers, 5 FP4 with
 *          64 x 64 per wave and operands staged through LDS whatever the size
 *   key 10 K-split waves of the latter kernel, key 11 = 2: its partial tiles cross LDS as fp32
 *          even where fp16 pairs would be exact, key 12 rows of tiles per band of its tile order
 *          (automatic: 16), key 13 = 1: never its form with 128 x 64 of C per wave, 2: that form
 *          wherever it exists (xnor products without a K split, int32 or fp32 results)
 *   key 14 = 1: the short-K matrix-core convolution kernel fetches pixel words 8 bytes at a time
 *          even where 16 would do; 2: 16 at a time, but never in the form for channel-word
 *          counts that are multiples of four; 3: never in the form that holds one block per wave
 *   key 15 = 1: bmx_binary_fc never takes its one-launch form for very small layers
 *   key 8  K-split waves, key 9  tile variant (1: 32 x 32, 2: 64 x 64 per wave) of the matrix-core
 *          kernels */
int bmx_tune_set(int key, int value);

/* Measurement hooks (not part of the layers the paper defines).
 * bmx_last_kernel: name, template arguments and launch shape of the last compute kernel the
 *   calling thread launched through this library ("" before the first); a static buffer
 *   overwritten by the thread's next call.  Benchmarks label their figures with it.
 * bmx_probe_valu: a register-only chain of v_xor_b32 + v_bcnt_u32_b32 pairs (the inner loop of
 *   the xor/popcount kernels with nothing around it), `workgroups` workgroups of 256 lanes, each
 *   lane 128 * iters pairs, i.e. workgroups * 256 * iters * 128 * 64 binary operations per
 *   launch.  Timed by the caller, it gives the VALU xor+popcount peak actually reachable; the
 *   first wave also writes out3[0] = shader clock cycles and out3[1] = constant-rate wall clock
 *   ticks (*wall_clock_khz per millisecond) it spent in the chain, whose ratio is the shader
 *   clock observed under load.  out3: device, 3 x uint64, 8-byte aligned. */
const char* bmx_last_kernel(void);
int bmx_probe_valu(int workgroups, int iters, unsigned long long* out3, int* wall_clock_khz, void* stream);

/* Static, human-readable name of a status code. */
const char* bmx_status_string(int status);

/* Library version, major * 10000 + minor * 100 + patch. */
int bmx_version(void);

#ifdef __cplusplus
}
#endif
#endif /* BMX_H */
