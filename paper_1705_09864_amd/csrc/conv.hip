// Implicit-GEMM binary convolution on the channel-packed, halo-padded image.
// Paper: Sec. 3.1 (M = filters, N = batch * output pixels, K = kh * kw * C).  The im2col
// matrix is never formed.
//
// Data layout.  The activation pack writes Xp [N][H + 2*pad][W + 2*pad][Cw] uint64, pixel
// (h, w) at row h + pad, column w + pad.  The halo holds the constant word "every real
// channel = +1": the float image is zero padded before the sign function and sign(0) = +1,
// so a padded tap is a +1 for every channel.  With the halo in memory the convolution
// gathers taps without any bounds test: the address of tap (kh, kw), word cw of output
// pixel (n, ho, wo) is  base(n, ho, wo) + (kh * Wp + kw) * Cw + cw  with a wave-uniform
// offset.
//
// Kernel shape.  Lanes span 64 consecutive output pixels (flat over n, ho, wo), so the NCHW
// stores are coalesced.  A lane keeps its whole K (KW uint64 words = taps * Cw) in VGPRs
// ("B stationary") and the wave streams filter rows past it: the row is wave-uniform, lives
// in SGPRs (scalar loads) and enters v_xor_b32 as the scalar operand, so the inner loop is
// nothing but v_xor_b32 + v_bcnt_u32_b32 (the popcount instruction also accumulates).
#include "bmx_internal.h"
#include "scalar_stream.h"

namespace bmx {

namespace {

constexpr int kMaxStationaryWords = 36;

struct ConvParams {
  const uint64_t* Xp;   // halo-padded packed image
  const uint32_t* Wp;   // [O][ld] words as dwords, KW data words per row
  int row_pad_dw;       // dwords between the end of a row's data and the next row
  const float* alpha;   // [O] or null
  int32_t* out_i32;
  float* out_f32;
  int64_t P;            // N * Ho * Wo
  int O, HoWo, Wo, Hp, Wp_pix, Cw, stride, Kreal, cn;  // cn: filters per wave
  FastDiv div_howo, div_wo;
  int off[kMaxStationaryWords];  // word offset of K-word j relative to the pixel base
};

// A filter row of 2*KW dwords is consumed in NSEG segments of SEG dwords; two SGPR buffers
// alternate so that the scalar loads of the next segment are in flight while the VALU works
// through the current one.
template <int KW>
struct SegShape {
  static constexpr int kDwords = 2 * KW;
  static constexpr int kNseg = (kDwords + 31) / 32;
  static constexpr int kSeg = kDwords / kNseg;
  static_assert(kSeg * kNseg == kDwords, "row must split into equal segments");
};

// FRESH: the segment opens a row, so its first popcount starts the count instead of adding.
template <int SEG, bool FRESH, int J = 0>
__device__ __forceinline__ int seg_popcount(const ScalarSeg<SEG>& a, const uint32_t* b, int pc) {
  if constexpr (J < SEG) {
    const int c = __builtin_popcount(b[J] ^ a.template get<J>());
    pc = (FRESH && J == 0) ? c : pc + c;
    asm volatile("" : "+v"(pc));  // keep the xor / popcount-accumulate chain as written
    return seg_popcount<SEG, FRESH, J + 1>(a, b, pc);
  } else {
    return pc;
  }
}

enum ConvOut { kOutI32 = 0, kOutF32 = 1, kOutF32Alpha = 2 };

// Every kernel argument the wave is going to need, consumed by empty asm statements at the
// top of the kernel: the compiler then requests all of them in one batch of scalar loads
// and waits once, instead of paying one memory round trip per group of first uses.
template <int KW, int J = 0>
__device__ __forceinline__ void touch_offsets(const ConvParams& p) {
  if constexpr (J + 4 <= KW) {
    asm volatile("" ::"s"(p.off[J]), "s"(p.off[J + 1]), "s"(p.off[J + 2]), "s"(p.off[J + 3]));
    touch_offsets<KW, J + 4>(p);
  } else if constexpr (J < KW) {
    asm volatile("" ::"s"(p.off[J]));
    touch_offsets<KW, J + 1>(p);
  }
}
template <int KW>
__device__ __forceinline__ void touch_args(const ConvParams& p) {
  asm volatile("" ::"s"(p.Xp), "s"(p.Wp), "s"(p.alpha), "s"(p.out_i32), "s"(p.out_f32), "s"(p.P),
               "s"(p.O), "s"(p.HoWo), "s"(p.Wo), "s"(p.Hp), "s"(p.Wp_pix), "s"(p.Cw), "s"(p.stride),
               "s"(p.Kreal), "s"(p.cn), "s"(p.row_pad_dw), "s"(p.div_howo.mul), "s"(p.div_howo.sh1), "s"(p.div_howo.sh2),
               "s"(p.div_wo.mul), "s"(p.div_wo.sh1), "s"(p.div_wo.sh2));
  if constexpr (KW <= 9) touch_offsets<KW>(p);  // longer tables would not stay in SGPRs anyway
}

template <int KW, int OUT>
__global__ void __launch_bounds__(256)
conv_stationary_kernel(const ConvParams p) {
  constexpr int SEG = SegShape<KW>::kSeg;
  constexpr int NSEG = SegShape<KW>::kNseg;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // Lanes (and whole waves of the last workgroup) past the last pixel repeat pixel P-1: they
  // compute and store the same values to the same addresses as the lane that owns it.  No
  // lane is ever masked off and there is no early exit, so every kernel argument can be
  // fetched in one batch at the top.
  touch_args<KW>(p);
  const int64_t pix = min(((int64_t)blockIdx.x * 4 + wave) * 64 + lane, p.P - 1);
  const uint32_t img = fast_div((uint32_t)pix, p.div_howo);
  const uint32_t rem = (uint32_t)pix - img * (uint32_t)p.HoWo;
  const uint32_t ho = fast_div(rem, p.div_wo);
  const uint32_t wo = rem - ho * (uint32_t)p.Wo;
  // Per-lane byte offsets are 32-bit and every base is wave-uniform, so loads and stores
  // use the scalar-base + vector-offset addressing form and need no vector address math.
  // (The host routes shapes whose packed image or per-wave output span exceed 4 GiB to the
  // general kernel.)
  const uint32_t xoff =
      (((img * (uint32_t)p.Hp + ho * (uint32_t)p.stride) * (uint32_t)p.Wp_pix + wo * (uint32_t)p.stride) *
       (uint32_t)p.Cw) * 8u;
  const char* xbase = (const char*)p.Xp;
  uint32_t b[2 * KW];
#pragma unroll
  for (int j = 0; j < KW; ++j) {
    const uint32_t voff = xoff + (uint32_t)p.off[j] * 8u;  // one 32-bit add per tap
    const uint64_t v = *(const uint64_t*)(xbase + voff);
    b[2 * j] = (uint32_t)v;
    b[2 * j + 1] = (uint32_t)(v >> 32);
  }
  const int o0 = blockIdx.y * p.cn;
  const int nrows = min(p.cn, p.O - o0);
  // alpha of the wave's filters: filter o0 + i in lane i (at most 64 filters per wave), handed
  // out with readlane as a row completes
  float alpha_lane = 1.0f;
  if (OUT == kOutF32Alpha) alpha_lane = p.alpha[o0 + min(lane, nrows - 1)];
  // Rows o0 .. o0+nrows-1 are a stream of nrows * NSEG segments (row_pad_dw dwords of
  // padding follow the last segment of every row).
  const int nseg_total = nrows * NSEG;
  const_u32_ptr stream = (const_u32_ptr)uniform_addr(
      (uint64_t)(uintptr_t)p.Wp + (int64_t)o0 * (4 * (2 * KW + p.row_pad_dw)));
  // output: uniform base of (image of lane 0, filter o0), advanced by one plane per row
  const uint32_t img0 = __builtin_amdgcn_readfirstlane(img);
  const uint32_t ooff = ((img - img0) * (uint32_t)p.O * (uint32_t)p.HoWo + rem) * 4u;
  char* obase = (char*)(OUT == kOutI32 ? (void*)p.out_i32 : (void*)p.out_f32) +
                ((int64_t)img0 * p.O + o0) * p.HoWo * 4;
  const int64_t ostride = (int64_t)p.HoWo * 4;

  ScalarSeg<SEG> buf[2];
  int pc = 0;
  const_u32_ptr src = stream;
  int left = nseg_total - 1;  // segments after the one at src
  buf[0].issue(src);
  for (int t = 0; t < nseg_total; t += 2 * NSEG) {  // two rows per trip
#pragma unroll
    for (int i = 0; i < 2 * NSEG; ++i) {
      const int cur = i & 1, nxt = cur ^ 1;
      const int seg_in_row = i % NSEG;
      const int row = t / NSEG + i / NSEG;  // row within the wave's range (uniform)
      // the following segment; past the end of this wave's stream the last segment is fetched
      // again, so nothing beyond the weights is ever read
      src += (left > 0) ? (SEG + (seg_in_row == NSEG - 1 ? p.row_pad_dw : 0)) : 0;
      left -= 1;
      buf[cur].landed(src);
      buf[nxt].issue(src);
      if (seg_in_row == 0) pc = seg_popcount<SEG, true>(buf[cur], b, pc);
      else pc = seg_popcount<SEG, false>(buf[cur], b + seg_in_row * SEG, pc);
      if (seg_in_row == NSEG - 1) {
        if (row < nrows) {
          int dot;  // K - 2 * popcount in one VALU op (both operands are below 2^23)
          asm("v_mad_i32_i24 %0, %1, -2, %2" : "=v"(dot) : "v"(pc), "s"(p.Kreal));
          // scalar base + 32-bit lane offset: the store needs no vector address arithmetic
          // (non-temporal: the output is written once and never read here; measured 6.5
          // against 7.8 us on the 16 x 64 x 56 x 56 layer)
          if (OUT == kOutF32Alpha) {
            const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, alpha_lane), row));
            const float v = a * (float)dot;
            asm volatile("global_store_dword %0, %1, %2 nt" ::"v"(ooff), "v"(v), "s"(obase) : "memory");
          } else if (OUT == kOutF32) {
            const float v = (float)dot;
            asm volatile("global_store_dword %0, %1, %2 nt" ::"v"(ooff), "v"(v), "s"(obase) : "memory");
          } else {
            asm volatile("global_store_dword %0, %1, %2 nt" ::"v"(ooff), "v"(dot), "s"(obase) : "memory");
          }
        }
        obase += ostride;
      }
    }
  }
}

// General shape: any number of K words, one thread per output, taps addressed with the
// same halo trick.  Only for images too large for the 32-bit offsets of the other two paths.
__global__ void __launch_bounds__(256)
conv_general_kernel(const uint64_t* __restrict__ Xp, const uint64_t* __restrict__ Wp,
                    const float* __restrict__ alpha, int32_t* __restrict__ out_i32,
                    float* __restrict__ out_f32, int64_t P, int O, int HoWo, int Wo, int Hp,
                    int Wp_pix, int Cw, int stride, int KH, int KWid, int Kreal, int ld_words,
                    FastDiv div_howo, FastDiv div_wo) {
  const int64_t pix = (int64_t)blockIdx.x * 64 + (threadIdx.x & 63);
  const int o = blockIdx.y * 4 + (threadIdx.x >> 6);
  if (pix >= P || o >= O) return;
  const uint32_t img = fast_div((uint32_t)pix, div_howo);
  const uint32_t rem = (uint32_t)pix - img * (uint32_t)HoWo;
  const uint32_t ho = fast_div(rem, div_wo);
  const uint32_t wo = rem - ho * (uint32_t)Wo;
  const uint64_t* xb = Xp + (((int64_t)img * Hp + ho * stride) * Wp_pix + wo * stride) * Cw;
  const uint64_t* wrow = Wp + (int64_t)o * ld_words;
  int pc = 0;
  for (int kh = 0; kh < KH; ++kh)
    for (int kw = 0; kw < KWid; ++kw) {
      const uint64_t* xp = xb + ((int64_t)kh * Wp_pix + kw) * Cw;
      const uint64_t* wp = wrow + (kh * KWid + kw) * Cw;
      for (int cw = 0; cw < Cw; ++cw) pc += __popcll(xp[cw] ^ wp[cw]);
    }
  const int dot = Kreal - 2 * pc;
  const int64_t idx = ((int64_t)img * O + o) * HoWo + rem;
  if (out_i32) out_i32[idx] = dot;
  else out_f32[idx] = (alpha ? alpha[o] : 1.0f) * (float)dot;
}

template <int KW>
void launch_stationary(const ConvParams& p, int64_t groups, int cblocks, hipStream_t s) {
  dim3 grid((unsigned)ceil_div(groups, 4), (unsigned)cblocks);
  note_kernel("conv_stationary_kernel<%d,%s> grid %u x %u x 256, %d filters per wave", KW,
              p.out_f32 ? (p.alpha ? "f32*alpha" : "f32") : "i32", grid.x, grid.y, p.cn);
  if (p.out_f32 && p.alpha)
    hipLaunchKernelGGL((conv_stationary_kernel<KW, kOutF32Alpha>), grid, dim3(256), 0, s, p);
  else if (p.out_f32)
    hipLaunchKernelGGL((conv_stationary_kernel<KW, kOutF32>), grid, dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL((conv_stationary_kernel<KW, kOutI32>), grid, dim3(256), 0, s, p);
}

}  // namespace

FastDiv make_fast_div(uint32_t d) {
  FastDiv f;
  uint32_t s = 0;
  while (((uint64_t)1 << s) < d) ++s;  // s = ceil(log2 d)
  f.mul = (uint32_t)((((uint64_t)1 << 32) * (((uint64_t)1 << s) - d)) / d + 1);
  f.sh1 = s < 1 ? s : 1;
  f.sh2 = s < 1 ? 0 : s - 1;
  return f;
}

int conv_filters_per_wave = 0;  // 0 = automatic; settable for tuning sweeps
int conv_path = 0;              // 0 = automatic, 1 = stationary, 2 = GEMM kernel, 3 = general
int conv_ws_x4 = 0;             // 1 = the short-K matrix-core kernel never fetches pixel words 16 bytes at a time; 2 = never in its form for runs of four channel words; 3 = never in its form with one block per wave

hipError_t launch_binary_conv2d(const uint64_t* Xp, int N, int C, int H, int W, const uint64_t* Wp,
                                int O, int KH, int KW, int stride, int pad, const float* alpha,
                                int32_t* out_i32, float* out_f32, hipStream_t s) {
  const int Ho = (H + 2 * pad - KH) / stride + 1;
  const int Wo = (W + 2 * pad - KW) / stride + 1;
  const int Cw = (int)words_for(C);
  const int64_t P = (int64_t)N * Ho * Wo;
  const int Hp = H + 2 * pad, Wpp = W + 2 * pad;
  const int kwords = KH * KW * Cw;
  const int ld_words = (int)conv_weight_row_words(kwords);
  const FastDiv d1 = make_fast_div((uint32_t)(Ho * Wo)), d2 = make_fast_div((uint32_t)Wo);
  const int64_t groups = ceil_div(P, 64);
  // both fast kernels address the packed image with 32-bit byte offsets from a uniform base
  // (the stationary kernel also a wave's output span)
  const bool image32 = (int64_t)N * Hp * Wpp * Cw * 8 < ((int64_t)1 << 32);
  const bool fits32 = image32 && (int64_t)(64 / (Ho * Wo) + 2) * O * Ho * Wo * 4 < ((int64_t)1 << 32);
  const bool stationary_ok =
      fits32 && (kwords == 1 || kwords == 2 || kwords == 4 || kwords == 9 || kwords == 18 ||
                 kwords == 25 || kwords == 27 || kwords == 36);
  // Of the popcount kernels the stationary one (whole K in registers, no accumulators) is the
  // faster on every shape it can hold; a K beyond 36 words goes to the popcount GEMM kernel,
  // which splits K and rows.
  int path = conv_path;
  if (path == 4 || path == 5 || path == 6) path = 0;
  if (path == 1 && !stationary_ok) path = 0;
  if (path == 2 && !image32) path = 0;
  if (path == 0) path = stationary_ok ? 1 : (image32 ? 2 : 3);
  // K of 9, 18, 25, 27, 36, 49 or 50 words: the matrix-core kernel with the expanded filters in LDS.
  // Measured with inputs and outputs rotating through HBM, against the stationary kernel:
  // 6.4 against 6.7 us on 16 x 64 x 56 x 56 -> 64 filters, 17.0 against 24.4 us on four times
  // the batch, 9.6 against 10.9 us on 8 x 64 x 56 x 56 -> 256, 6.3 against 7.9 us on
  // 16 x 128 x 28 x 28 -> 128; at 36 words 15.6 against 16.8 us for the GEMM-shaped matrix-core
  // kernel (64 x 256 x 14 x 14 -> 256) and 8.2 against 8.6 us at stride 2.
  // The GEMM kernel with 64 x 64 per wave and LDS-staged operands in its convolution form (6
  // forces it): the choice beyond the 50 words the short-K kernel reaches, given an even number
  // of channel words.  Measured per call against the 32 x 32 per wave matrix-core kernel, inputs
  // from HBM: 200 x 256 x 12 x 12, 5 x 5, 64 filters 16.0 against 19.3 us, 512 channels 25.2
  // against 30.8 us, 7 x 7 over 256 channels 20.5 against 26.3 us.  Within the short-K kernel's
  // reach it wins only where that kernel cannot fill the chip (64 x 256 x 14 x 14 at stride 2: 6.5
  // against 7.1 us) and loses where the output is large (stride 1: 12.8 against 11.2 us: its
  // tiles store all at once at the end, the short-K kernel block by block), so it is not chosen there.
  if (conv_path == 6 || (conv_path == 0 && kwords > 50 && (Cw & 1) == 0)) {
    hipError_t err = hipSuccess;
    if (launch_conv_fp4(Xp, N, C, H, W, Wp, O, KH, KW, stride, pad, alpha, out_i32, out_f32, s, &err)) return err;
  }
  if ((conv_path == 5 || (conv_path == 0 && conv_weight_short_k(kwords))) && gemm_engine != 1) {
    hipError_t err = hipSuccess;
    if (launch_conv_mfma_ws(Xp, N, C, H, W, Wp, O, KH, KW, stride, pad, alpha, out_i32, out_f32, nullptr, nullptr, 0,
                            s, &err))
      return err;
  }
  if (conv_path == 4 || (conv_path == 0 && (!stationary_ok || kwords >= 36))) {
    // From K = 36 words (3 x 3 over 256 channels) on, the matrix cores: measured 15.7 against
    // 18.6 us on 64 x 256 x 14 x 14 -> 256 filters, 7.8 against 10.2 us on its stride-2 twin,
    // and 1.4 to 2.3 times faster than the xor/popcount GEMM kernel beyond the stationary
    // kernel's reach (5 x 5 kernels over 128 .. 512 channels).  Below that (18 words: 8.8
    // against 7.9 us; 9 words: 11.1 against 8.3 us) the stationary kernel stays ahead.
    hipError_t err = hipSuccess;
    if (launch_conv_mfma(Xp, N, C, H, W, Wp, O, KH, KW, stride, pad, alpha, out_i32, out_f32, s, &err))
      return err;
  }
  if (path == 2)
    return launch_conv_gemm(Xp, N, C, H, W, Wp, O, KH, KW, stride, pad, alpha, out_i32, out_f32, s);
  if (path == 1) {
    ConvParams p;
    p.Xp = Xp;
    p.Wp = (const uint32_t*)Wp;
    p.row_pad_dw = 2 * (ld_words - kwords);
    p.alpha = alpha;
    p.out_i32 = out_i32;
    p.out_f32 = out_f32;
    p.P = P;
    p.O = O;
    p.HoWo = Ho * Wo;
    p.Wo = Wo;
    p.Hp = Hp;
    p.Wp_pix = Wpp;
    p.Cw = Cw;
    p.stride = stride;
    p.Kreal = C * KH * KW;
    p.div_howo = d1;
    p.div_wo = d2;
    for (int j = 0; j < kMaxStationaryWords; ++j) p.off[j] = 0;
    for (int kh = 0; kh < KH; ++kh)
      for (int kw = 0; kw < KW; ++kw)
        for (int cw = 0; cw < Cw; ++cw)
          p.off[(kh * KW + kw) * Cw + cw] = (kh * Wpp + kw) * Cw + cw;
    // Filters per wave.  A wave pays its gather once and then streams cn filter rows, so
    // more filters per wave amortise the gather better (below 8 the gather dominates), but
    // the grid should still fill the chip.  The 36-word kernel holds 88 VGPRs, i.e. five
    // waves per SIMD: a grid of at most 5 * 1024 waves is resident at once, and sweeps of the
    // ResNet-stage shapes put the optimum at the smallest even cn >= 8 that gets there (a
    // grid slightly over it pays a second, mostly empty round; the kernel consumes rows in
    // pairs, so an odd count costs a row that is computed and dropped).
    int cn = conv_filters_per_wave;
    if (cn <= 0) {
      cn = 8;
      while (cn < O && cn < 64 && groups * ceil_div(O, cn) > 5 * 1024) cn += 2;
    }
    if (cn > 64) cn = 64;  // the kernel keeps a wave's alphas one per lane
    p.cn = cn;
    const int cblocks = (int)ceil_div(O, cn);
    switch (kwords) {
      case 1: launch_stationary<1>(p, groups, cblocks, s); break;
      case 2: launch_stationary<2>(p, groups, cblocks, s); break;
      case 4: launch_stationary<4>(p, groups, cblocks, s); break;
      case 9: launch_stationary<9>(p, groups, cblocks, s); break;
      case 18: launch_stationary<18>(p, groups, cblocks, s); break;
      case 25: launch_stationary<25>(p, groups, cblocks, s); break;
      case 27: launch_stationary<27>(p, groups, cblocks, s); break;
      default: launch_stationary<36>(p, groups, cblocks, s); break;
    }
    return hipGetLastError();
  }
  dim3 grid((unsigned)groups, (unsigned)ceil_div(O, 4));
  note_kernel("conv_general_kernel grid %u x %u x 256", grid.x, grid.y);
  hipLaunchKernelGGL(conv_general_kernel, grid, dim3(256), 0, s, Xp, Wp, alpha, out_i32, out_f32, P,
                     O, Ho * Wo, Wo, Hp, Wpp, Cw, stride, KH, KW, C * KH * KW, ld_words, d1, d2);
  return hipGetLastError();
}

}  // namespace bmx
