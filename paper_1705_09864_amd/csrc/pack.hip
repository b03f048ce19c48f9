// Binarise / quantise + bit-pack kernels (HBM-bandwidth bound).
// Paper: Sec. 1 (sign binarisation, 64 values per word), Sec. 3.1 (the per-forward
// input binarisation step), Sec. 2.1 Eq. 1 (k-bit quantiser).
#include "bmx_internal.h"

namespace bmx {

static constexpr int kWave = 64;

// Row pack.  A wave packs segments of 16 consecutive words (1024 floats) of one row: lane
// <-> k, so every load instruction is a 256-byte coalesced read and the 64-lane compare
// mask is the packed word itself.  All 16 loads of a segment are issued before the first
// compare.  A workgroup owns one contiguous stretch of the segment list (its four waves
// interleave inside it).  Inputs larger than the memory-side cache are read with non-temporal
// loads and 32-word segments: on a 2 GiB read, contiguous stretches + non-temporal loads
// measured 7.0 TB/s against 5.3-5.8 TB/s for cached loads walking the list with a grid stride;
// on inputs that fit the caches (activations from the previous layer) the same loads lose.
constexpr int kSegWords = 16;

template <int kSegWords, bool NT>
__device__ __forceinline__ void pack_row_segments(const float* __restrict__ x, int64_t rows,
                                                  int64_t cols, int64_t ldx,
                                                  uint64_t* __restrict__ out, int64_t out_ld,
                                                  int64_t Kw, int64_t segs_per_row,
                                                  int64_t first_block, int64_t per) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave, waves = blockDim.x / kWave;
  const int64_t total = rows * segs_per_row;
  const int64_t end = (first_block + 1) * per < total ? (first_block + 1) * per : total;
  for (int64_t seg = first_block * per + wave; seg < end; seg += waves) {
    const int64_t r = segs_per_row == total ? 0 : seg / segs_per_row;
    const int64_t b = seg - r * segs_per_row;
    const float* xr = x + r * ldx;
    const int64_t k0 = b * (64 * kSegWords) + lane;
    float v[kSegWords];
    if (k0 - lane + 64 * kSegWords <= cols) {  // whole segment inside the row (wave-uniform)
#pragma unroll
      for (int j = 0; j < kSegWords; ++j) v[j] = NT ? __builtin_nontemporal_load(xr + k0 + 64 * j) : xr[k0 + 64 * j];
    } else {
#pragma unroll
      for (int j = 0; j < kSegWords; ++j) {
        const int64_t k = k0 + 64 * j;
        v[j] = (k < cols) ? xr[k] : -1.0f;  // out-of-row lanes contribute 0 bits
      }
    }
    uint64_t mine = 0;
#pragma unroll
    for (int j = 0; j < kSegWords; ++j) {
      const uint64_t m = __ballot(v[j] >= 0.0f);
      if (lane == j) mine = m;
    }
    const int64_t w = b * kSegWords + lane;
    if (lane < kSegWords && w < Kw) out[r * out_ld + w] = mine;
  }
}

template <int SEG, bool NT>
__global__ void __launch_bounds__(256)
pack_rows_kernel(const float* __restrict__ x, int64_t rows, int64_t cols, int64_t ldx,
                 uint64_t* __restrict__ out, int64_t out_ld, int64_t Kw, int64_t segs_per_row,
                 int64_t segs_per_block) {
  pack_row_segments<SEG, NT>(x, rows, cols, ldx, out, out_ld, Kw, segs_per_row, (int64_t)blockIdx.x,
                             segs_per_block);
}

static void launch_pack_rows_grid(const float* x, int64_t rows, int64_t cols, int64_t ldx,
                                  uint64_t* out, int64_t out_ld, int64_t words_per_row,
                                  hipStream_t s) {
  const int64_t cap = 256 * 8;  // 8 workgroups of 4 waves per CU
  if (rows * cols * 4 > ((int64_t)256 << 20)) {  // beyond the 256 MB memory-side cache
    const int64_t spr = ceil_div(words_per_row, 32);
    int64_t blocks = ceil_div(rows * spr, 4);
    blocks = blocks < cap ? blocks : cap;
    note_kernel("pack_rows_kernel<32,nontemporal> grid %lld x 256", (long long)blocks);
    hipLaunchKernelGGL((pack_rows_kernel<32, true>), dim3((unsigned)blocks), dim3(256), 0, s, x, rows, cols, ldx,
                       out, out_ld, words_per_row, spr, ceil_div(rows * spr, blocks));
    return;
  }
  const int64_t spr = ceil_div(words_per_row, kSegWords);
  int64_t blocks = ceil_div(rows * spr, 4);
  blocks = blocks < cap ? blocks : cap;
  note_kernel("pack_rows_kernel<16,cached> grid %lld x 256", (long long)blocks);
  hipLaunchKernelGGL((pack_rows_kernel<kSegWords, false>), dim3((unsigned)blocks), dim3(256), 0, s, x, rows, cols,
                     ldx, out, out_ld, words_per_row, spr, ceil_div(rows * spr, blocks));
}

hipError_t launch_pack_rows(const float* x, int64_t rows, int64_t cols, int64_t ldx, uint64_t* out,
                            int64_t out_ld, hipStream_t s) {
  const int64_t Kw = words_for(cols);
  // A dense matrix whose rows are whole words is one long row.
  if (ldx == cols && out_ld == Kw && (cols % 64) == 0) {
    cols = rows * cols;
    ldx = cols;
    rows = 1;
    out_ld = cols / 64;
  }
  launch_pack_rows_grid(x, rows, cols, ldx, out, out_ld, words_for(cols), s);
  return hipGetLastError();
}

// Row pack into rows of out_ld words, writing every word of a row (zeros past the last
// data word): the chunk-padded activation rows read by the scalar side of the GEMM kernel.
hipError_t launch_pack_rows_padded(const float* x, int64_t rows, int64_t cols, int64_t ldx,
                                   uint64_t* out, int64_t out_ld, hipStream_t s) {
  launch_pack_rows_grid(x, rows, cols, ldx, out, out_ld, out_ld, s);
  return hipGetLastError();
}

// Inverse of the row pack: element k of row r -> +1.0f / -1.0f (a stored 1-bit model back
// to the float weights every pack routine starts from, Sec. 2.2.3).  A wave per word, lane =
// bit; grid-stride over the words.
__global__ void __launch_bounds__(256)
unpack_pm1_kernel(const uint64_t* __restrict__ bits, int64_t rows, int64_t K, int64_t ld_words,
                  float* __restrict__ out, int64_t ldo) {
  const int lane = threadIdx.x & 63;
  const int64_t Kw = words_for(K);
  const int64_t total = rows * Kw;
  for (int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); i < total; i += (int64_t)gridDim.x * 4) {
    const int64_t r = i / Kw, w = i - r * Kw;
    const int64_t k = w * 64 + lane;
    const uint64_t word = bits[r * ld_words + w];
    if (k < K) out[r * ldo + k] = ((word >> lane) & 1) ? 1.0f : -1.0f;
  }
}

hipError_t launch_unpack_pm1(const uint64_t* bits, int64_t rows, int64_t K, int64_t ld_words, float* out,
                             int64_t ldo, hipStream_t s) {
  const int64_t blocks = ceil_div(rows * words_for(K), 4);
  hipLaunchKernelGGL(unpack_pm1_kernel, dim3((unsigned)(blocks < 65536 ? blocks : 65536)), dim3(256), 0, s, bits,
                     rows, K, ld_words, out, ldo);
  return hipGetLastError();
}

// Rows of 32-bit words (the 32-bit BINARY_WORD flavour of Sec. 2.2.1) -> rows of 64-bit words:
// word w of a row is dwords 2w (low half) and 2w + 1 (high half, zero when the row has an odd
// number of dwords).  With bits LSB first and little-endian words this moves no bit: element k
// is bit k % 32 of dword k / 32 and bit k % 64 of word k / 64 alike.  One thread per word.
__global__ void __launch_bounds__(256)
widen_words32_kernel(const uint32_t* __restrict__ in, int64_t rows, int64_t Kd, int64_t ld_dw,
                     uint64_t* __restrict__ out, int64_t out_ld) {
  const int64_t Kw = (Kd + 1) / 2;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= rows * Kw) return;
  const int64_t r = i / Kw, w = i - r * Kw;
  const uint32_t* row = in + r * ld_dw;
  const uint32_t lo = row[2 * w];
  const uint32_t hi = 2 * w + 1 < Kd ? row[2 * w + 1] : 0u;
  out[r * out_ld + w] = ((uint64_t)hi << 32) | lo;
}

hipError_t launch_widen_words32(const uint32_t* in, int64_t rows, int64_t K, int64_t ld_dw, uint64_t* out,
                                int64_t out_ld, hipStream_t s) {
  const int64_t Kd = (K + 31) / 32;
  const int64_t total = rows * ((Kd + 1) / 2);
  hipLaunchKernelGGL(widen_words32_kernel, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, s, in, rows, Kd,
                     ld_dw, out, out_ld);
  return hipGetLastError();
}

// Strided pack (the matrix is stored K x ncol, pack down the columns): a wave packs one
// word of 64 consecutive columns: lanes span columns, so every load instruction is a
// coalesced 256-byte read of one K row, and all 64 row loads of a lane are issued before
// the first compare.  The word is assembled in two 32-bit halves.
__global__ void __launch_bounds__(256)
pack_strided_kernel(const float* __restrict__ x, int64_t batch, int64_t K, int64_t ncol,
                    int64_t ldx, int64_t batch_stride, uint64_t* __restrict__ out, int64_t out_ld,
                    int64_t Kw, int64_t col_groups) {
  const int lane = threadIdx.x & 63;
  const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x / kWave);
  const int64_t total = batch * Kw * col_groups;
  for (int64_t item = (int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave);
       item < total; item += nwaves) {
    const int64_t g = item % col_groups;
    const int64_t t = item / col_groups;
    const int64_t w = t % Kw;
    const int64_t b = t / Kw;
    const int64_t n = g * 64 + lane;
    const int64_t nc = n < ncol ? n : ncol - 1;
    const float* xb = x + b * batch_stride + (w * 64) * ldx + nc;
    const int64_t kmax = K - w * 64;  // rows left in this word (>= 1)
    float v[64];
    if (kmax >= 64) {
#pragma unroll
      for (int j = 0; j < 64; ++j) v[j] = xb[(int64_t)j * ldx];
    } else {
#pragma unroll
      for (int j = 0; j < 64; ++j) v[j] = (j < kmax) ? xb[(int64_t)j * ldx] : -1.0f;
    }
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) lo |= (v[j] >= 0.0f ? 1u : 0u) << j;
#pragma unroll
    for (int j = 0; j < 32; ++j) hi |= (v[32 + j] >= 0.0f ? 1u : 0u) << j;
    if (n < ncol) out[(b * ncol + n) * out_ld + w] = ((uint64_t)hi << 32) | lo;
  }
}

hipError_t launch_pack_strided(const float* x, int64_t batch, int64_t K, int64_t ncol, int64_t ldx,
                               int64_t batch_stride, uint64_t* out, int64_t out_ld, hipStream_t s) {
  const int64_t Kw = words_for(K);
  const int64_t groups = ceil_div(ncol, 64);
  const int64_t blocks = ceil_div(batch * Kw * groups, 4);
  const int64_t cap = 256 * 6;  // the kernel holds 64 loaded values per lane: 6 waves per SIMD
  note_kernel("pack_strided_kernel grid %lld x 256", (long long)(blocks < cap ? blocks : cap));
  hipLaunchKernelGGL(pack_strided_kernel, dim3((unsigned)(blocks < cap ? blocks : cap)), dim3(256), 0,
                     s, x, batch, K, ncol, ldx, batch_stride, out, out_ld, Kw, groups);
  return hipGetLastError();
}

// NCHW channel pack.  A wave packs 64 consecutive pixels of one image for one 64-channel
// word: lanes span pixels, so every load instruction is a coalesced 256-byte read of one
// channel plane, and all 64 channel loads of a lane are issued before the first compare
// (16 KiB in flight per wave).  The word is assembled in two 32-bit halves.  Workgroup 0 of
// every (image, word) also writes the constant halo words.  The image is read exactly once, so
// the loads are non-temporal (they do not displace what the convolution that follows needs:
// 12.8 us against 13.4 us per configuration-2 layer with the input coming from HBM).
// THR: bit = (value >= thr[channel]) instead of (value >= 0): the packing behind a layer whose
// sign decision carries a folded per-channel threshold.
template <bool THR>
__global__ void __launch_bounds__(256)
pack_nchw_kernel(const float* __restrict__ x, int C, int HW, int W, int pad, int Hp, int Wp, int Cw,
                 const float* __restrict__ thr, uint64_t* __restrict__ xp) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int cw = blockIdx.y;
  const int n = blockIdx.z;
  const int p = (blockIdx.x * 4 + wave) * 64 + lane;
  uint64_t* xpn = xp + (int64_t)n * Hp * Wp * Cw;
  if (p - lane < HW) {  // wave-uniform: this 64-pixel group exists
    const int pc = p < HW ? p : HW - 1;
    const int c0 = cw * 64;
    const float* xb = x + ((int64_t)n * C + c0) * HW + pc;
    float v[64];
    if (c0 + 64 <= C) {
#pragma unroll
      for (int j = 0; j < 64; ++j) v[j] = __builtin_nontemporal_load(xb + (int64_t)j * HW);
    } else {
#pragma unroll
      for (int j = 0; j < 64; ++j) v[j] = (c0 + j < C) ? xb[(int64_t)j * HW] : -1.0f;
    }
    uint32_t lo = 0, hi = 0;
    if constexpr (THR) {
      // (missing channels hold -1 and compare against 0)
#pragma unroll
      for (int j = 0; j < 32; ++j) lo |= (v[j] >= (c0 + j < C ? thr[c0 + j] : 0.0f) ? 1u : 0u) << j;
#pragma unroll
      for (int j = 0; j < 32; ++j) hi |= (v[32 + j] >= (c0 + 32 + j < C ? thr[c0 + 32 + j] : 0.0f) ? 1u : 0u) << j;
    } else {
#pragma unroll
      for (int j = 0; j < 32; ++j) lo |= (v[j] >= 0.0f ? 1u : 0u) << j;
#pragma unroll
      for (int j = 0; j < 32; ++j) hi |= (v[32 + j] >= 0.0f ? 1u : 0u) << j;
    }
    if (p < HW) {
      const int h = p / W, w = p - h * W;
      xpn[((int64_t)(h + pad) * Wp + (w + pad)) * Cw + cw] = ((uint64_t)hi << 32) | lo;
    }
  }
  if (pad > 0 && blockIdx.x == 0) {
    const uint64_t ones = (cw == Cw - 1 && (C % 64)) ? (((uint64_t)1 << (C % 64)) - 1) : ~(uint64_t)0;
    const int H = HW / W;
    const int nh = Hp * Wp - HW;
    for (int i = threadIdx.x; i < nh; i += 256) {
      int hh, ww;
      if (i < pad * Wp) {
        hh = i / Wp;
        ww = i - hh * Wp;
      } else if (i < 2 * pad * Wp) {
        const int j = i - pad * Wp;
        hh = j / Wp;
        ww = j - hh * Wp;
        hh += pad + H;
      } else {
        const int j = i - 2 * pad * Wp;
        const int r = j / (2 * pad), c = j - r * (2 * pad);
        hh = pad + r;
        ww = c < pad ? c : W + c;
      }
      xpn[((int64_t)hh * Wp + ww) * Cw + cw] = ones;
    }
  }
}

hipError_t launch_pack_nchw_thr(const float* x, int N, int C, int H, int W, int pad, const float* thr,
                                uint64_t* xp, hipStream_t s) {
  const int Cw = (int)words_for(C);
  const int HW = H * W;
  dim3 grid((unsigned)ceil_div(HW, 256), (unsigned)Cw, (unsigned)N);
  note_kernel("pack_nchw_kernel<%s> grid %u x %u x %u x 256", thr ? "thr" : "sign", grid.x, grid.y, grid.z);
  if (thr)
    hipLaunchKernelGGL(pack_nchw_kernel<true>, grid, dim3(256), 0, s, x, C, HW, W, pad, H + 2 * pad,
                       W + 2 * pad, Cw, thr, xp);
  else
    hipLaunchKernelGGL(pack_nchw_kernel<false>, grid, dim3(256), 0, s, x, C, HW, W, pad, H + 2 * pad,
                       W + 2 * pad, Cw, thr, xp);
  return hipGetLastError();
}

hipError_t launch_pack_nchw(const float* x, int N, int C, int H, int W, int pad, uint64_t* xp,
                            hipStream_t s) {
  return launch_pack_nchw_thr(x, N, C, H, W, pad, nullptr, xp, s);
}

// Offline weight packing for the convolution: one thread per word of the bit section.
// Wp[o][(kh*KW + kw)*Cw + cw] bit c = (w[o][64cw + c][kh][kw] >= 0); rows are ld words apart
// and the words between the data and ldb (the chunk-padded bit section) are written as zero.
// With consts set the row's K - 2 * popcount is summed with atomics into the float slot behind
// the bits, which the launcher's first kernel set to K.
__global__ void __launch_bounds__(256)
pack_conv_weights_kernel(const float* __restrict__ w, int O, int C, int KH, int KW, int Cw, int ld, int ldb,
                         int consts, uint64_t* __restrict__ Wp) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)O * ldb;
  if (idx >= total) return;
  const int64_t o = idx / ldb;
  const int j = (int)(idx - o * ldb);
  const int kwords = KH * KW * Cw;
  uint64_t word = 0;
  if (j < kwords) {
    const int cw = j % Cw;
    const int t = j / Cw;
    const int kw = t % KW;
    const int kh = t / KW;
    for (int c = 0; c < 64; ++c) {
      const int ch = cw * 64 + c;
      if (ch < C) {
        const float v = w[((o * C + ch) * KH + kh) * KW + kw];
        if (v >= 0.0f) word |= (uint64_t)1 << c;
      }
    }
  }
  uint64_t* row = Wp + o * ld;
  row[j] = word;
  if (consts && j < kwords)  // (integers below 2^24: the float sum is exact in any order)
    atomicAdd((float*)(row + ldb), -2.0f * (float)__popcll(word));
}

// The float slot of every row starts at K (C * KH * KW); the pad word behind it at zero.
__global__ void __launch_bounds__(256)
init_conv_weight_consts_kernel(int O, int ld, int ldb, int kwords, float K, uint64_t* __restrict__ Wp) {
  const int o = blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= O) return;
  uint32_t* c = (uint32_t*)(Wp + (int64_t)o * ld + ldb);
  c[0] = __float_as_uint(K);
  c[1] = c[2] = c[3] = 0;
}

hipError_t launch_pack_conv_weights(const float* w, int O, int C, int KH, int KW, uint64_t* Wp,
                                    hipStream_t s) {
  const int Cw = (int)words_for(C);
  const int kwords = KH * KW * Cw;
  const int ld = (int)conv_weight_row_words(kwords), ldb = (int)conv_weight_bits_words(kwords);
  const int consts = conv_weight_short_k(kwords) ? 1 : 0;
  if (consts)
    hipLaunchKernelGGL(init_conv_weight_consts_kernel, dim3((unsigned)ceil_div(O, 256)), dim3(256), 0, s, O, ld,
                       ldb, kwords, (float)((int64_t)C * KH * KW), Wp);
  const int64_t total = (int64_t)O * ldb;
  hipLaunchKernelGGL(pack_conv_weights_kernel, dim3((unsigned)ceil_div(total, 256)), dim3(256), 0, s,
                     w, O, C, KH, KW, Cw, ld, ldb, consts, Wp);
  return hipGetLastError();
}

// k-bit weights: T[m][n * bw + r] holds the 1-bit-weight form against weight plane r;
// S[m][n] = sum_r 2^r T[m][n * bw + r], out = float(S) / denom.
__global__ void __launch_bounds__(256)
quant_combine_kernel(const int32_t* __restrict__ T, int64_t M, int64_t N, int bw, float denom,
                     int32_t* __restrict__ S, float* __restrict__ out, int64_t ldo) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= M * N) return;
  const int64_t m = i / N, n = i - m * N;
  const int32_t* t = T + (m * N + n) * bw;
  int32_t acc = 0;
  for (int r = 0; r < bw; ++r) acc += t[r] << r;
  if (S) S[m * ldo + n] = acc;
  if (out) out[m * ldo + n] = (float)acc / denom;
}

hipError_t launch_quant_combine(const int32_t* T, int64_t M, int64_t N, int bw, float denom, int32_t* S,
                                float* out, int64_t ldo, hipStream_t s) {
  hipLaunchKernelGGL(quant_combine_kernel, dim3((unsigned)ceil_div(M * N, 256)), dim3(256), 0, s, T, M, N, bw,
                     denom, S, out, ldo);
  return hipGetLastError();
}

// alpha[r] = mean |w[r][:]|, one workgroup per row, fp64 accumulation.
__global__ void __launch_bounds__(256)
alpha_mean_abs_kernel(const float* __restrict__ w, int64_t rows, int64_t cols, int64_t ldw,
                      float* __restrict__ alpha) {
  __shared__ double part[256];
  for (int64_t r = blockIdx.x; r < rows; r += gridDim.x) {
    double acc = 0.0;
    for (int64_t j = threadIdx.x; j < cols; j += blockDim.x) acc += fabs((double)w[r * ldw + j]);
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) {
      if ((int)threadIdx.x < st) part[threadIdx.x] += part[threadIdx.x + st];
      __syncthreads();
    }
    if (threadIdx.x == 0) alpha[r] = (float)(part[0] / (double)cols);
    __syncthreads();
  }
}

hipError_t launch_alpha_mean_abs(const float* w, int64_t rows, int64_t cols, int64_t ldw,
                                 float* alpha, hipStream_t s) {
  const int64_t blocks = rows < 65535 * 16 ? rows : 65535 * 16;
  hipLaunchKernelGGL(alpha_mean_abs_kernel, dim3((unsigned)blocks), dim3(256), 0, s, w, rows, cols,
                     ldw, alpha);
  return hipGetLastError();
}

// Eq. 1 quantiser + bit-plane pack.  One workgroup per row m, lane <-> k: the four waves
// take every fourth segment of 16 words, and all 16 loads of a segment are issued before
// the first of them is used.  q = round(L * clamp(x)), ties away from zero, from the single
// fp32 product L * x.  Plane p of word w is the 64-lane mask of bit p of q and goes to row
// m * bits + p of `planes` (words up to ld_words are written, zeros past the data).  The row
// sum of q, needed by the plane GEMM epilogue, is reduced through LDS.
// The weight operand of the same GEMM is sign-packed by the workgroups past the first M of
// the same launch (wrows > 0), so that the two inputs cost one kernel launch, not two.
__global__ void __launch_bounds__(256)
quant_pack_kernel(const float* __restrict__ a, int64_t M, int64_t K, int64_t lda, int bits,
                  uint64_t* __restrict__ planes, int64_t ld_words, int32_t* __restrict__ rowsum,
                  const float* __restrict__ w, int64_t wrows, int64_t ldw,
                  uint64_t* __restrict__ wbits, int64_t wb_ld, int64_t wsegs_per_block, int affine) {
  __shared__ int32_t part[4];
  if ((int64_t)blockIdx.x >= M) {
    const int64_t Kw = words_for(K);
    pack_row_segments<kSegWords, false>(w, wrows, K, ldw, wbits, wb_ld, Kw, ceil_div(Kw, kSegWords),
                      (int64_t)blockIdx.x - M, wsegs_per_block);
    return;
  }
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int64_t m = blockIdx.x;
  const float L = (float)((1u << bits) - 1u);
  const float* ar = a + m * lda;
  uint64_t* prow = planes + m * bits * ld_words;
  int32_t sum = 0;
  for (int64_t w0 = (int64_t)wave * kSegWords; w0 < ld_words; w0 += 4 * kSegWords) {
    float v[kSegWords];
    if ((w0 + kSegWords) * 64 <= K) {
#pragma unroll
      for (int j = 0; j < kSegWords; ++j) v[j] = ar[(w0 + j) * 64 + lane];
      // (signed operand: [-1, 1] onto [0, 1] first, two fp32 operations)
      if (affine) {
#pragma unroll
        for (int j = 0; j < kSegWords; ++j) v[j] = __fmul_rn(__fadd_rn(v[j], 1.0f), 0.5f);
      }
    } else {
#pragma unroll
      for (int j = 0; j < kSegWords; ++j) {
        const int64_t k = (w0 + j) * 64 + lane;
        const float t = (k < K) ? ar[k] : 0.0f;
        v[j] = (affine && k < K) ? __fmul_rn(__fadd_rn(t, 1.0f), 0.5f) : t;
      }
    }
    int q[kSegWords];
#pragma unroll
    for (int j = 0; j < kSegWords; ++j) {
      q[j] = (int)roundf(__fmul_rn(L, fminf(fmaxf(v[j], 0.0f), 1.0f)));
      sum += q[j];
    }
    for (int p = 0; p < bits; ++p) {
      uint64_t mine = 0;
#pragma unroll
      for (int j = 0; j < kSegWords; ++j) {
        const uint64_t mask = __ballot((q[j] >> p) & 1);
        if (lane == j) mine = mask;
      }
      if (lane < kSegWords && w0 + lane < ld_words) prow[p * ld_words + w0 + lane] = mine;
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off, kWave);
  if (lane == 0) part[wave] = sum;
  __syncthreads();
  if (threadIdx.x == 0) rowsum[m] = part[0] + part[1] + part[2] + part[3];
}

hipError_t launch_quant_pack(const float* a, int64_t M, int64_t K, int64_t lda, int bits,
                             uint64_t* planes, int64_t ld_words, int32_t* rowsum, const float* w,
                             int64_t wrows, int64_t ldw, uint64_t* wbits, int64_t wb_ld,
                             hipStream_t s, bool affine) {
  int64_t wblocks = 0, per = 1;
  if (wrows > 0) {
    const int64_t segs = wrows * ceil_div(words_for(K), kSegWords);
    wblocks = ceil_div(segs, 4);
    if (wblocks > 256 * 8) wblocks = 256 * 8;
    per = ceil_div(segs, wblocks);
  }
  note_kernel("quant_pack_kernel grid %lld x 256", (long long)(M + wblocks));
  hipLaunchKernelGGL(quant_pack_kernel, dim3((unsigned)(M + wblocks)), dim3(256), 0, s, a, M, K, lda,
                     bits, planes, ld_words, rowsum, w, wrows, ldw, wbits, wb_ld, per, affine ? 1 : 0);
  return hipGetLastError();
}

}  // namespace bmx
