// Binary convolution on the FP4 matrix cores for short K (9, 18, 25, 27, 36,
// 49 or 50 words: 3 x 3, 5 x 5 and 7 x 7 filters over up to 256, 128 and 64 channels).
// Paper: Sec. 3.1 (M = filters, N = batch * output pixels, K = kh * kw * C), result
// out = alpha[o] * (K - 2 * popcount(filter xor patch)) (Sec. 2.2.2, Eq. 2).
//
// With the filter's bits read as f = +-1 and the patch's bits as x in {0, 1},
// K - 2 * pc(filter xor patch) = sum f (2 x - 1) = (K - 2 * pc(filter)) + 2 * sum f x: the sum on
// v_mfma_scale_f32_32x32x64_f8f6f4 with both operands FP4 (E2M1), the constant per filter
// (stored behind the filter's bits by the weight pack), and no popcount of the patch at all.
// A set pixel bit becomes a nibble worth 0.5, 1 or 2, a filter bit a nibble of the reciprocal
// magnitude whose sign bit is the inverted bit (see expand_pixel), so products are 0 or +-1
// and the fp32 sums exact integers.
//
// Shape.  A workgroup expands the bits of its 32 * TM filters into FP4 operands in LDS once
// (a few dozen VALU instructions per thread), and every MFMA step reads its A operand from
// there (16 bytes per lane), so filters cost no registers and no VALU work per pixel block.
// A wave walks over blocks of 32 output pixels: it fetches the pixels' KW words (one MFMA step
// of K = 64 consumes exactly one 64-bit word: lane (r, h) supplies half h of the word of pixel
// r), expands them (5 VALU instructions per word) and issues KW * TM
// MFMAs.  Lanes run along pixels (operand B), so the NCHW stores are two 128-byte runs per
// instruction.
#include <algorithm>
#include <type_traits>

#include "bmx_internal.h"

namespace bmx {

namespace {

typedef unsigned v2u __attribute__((ext_vector_type(2)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
// 16-byte accesses to the dword-typed LDS array: without may_alias the compiler is entitled to
// move the 32-bit accesses of the same memory across them (type-based alias analysis)
typedef v4i __attribute__((may_alias)) v4i_alias;

constexpr int kMaxWsWords = 50;

struct WsParams {
  const uint64_t* Xp;  // halo-padded packed image
  const uint32_t* Wp;  // [O][ld_dw] dwords: the filter's bits, at dword c0_dw the float K - 2 * popcount
  int ld_dw, c0_dw;
  const float* alpha;  // [O] or null
  int32_t* out_i32;
  float* out_f32;
  // packed-bit output (the next convolution's input image): [Nimg][oHp][oWp][oCw] words seen as
  // dwords, interior offset opad; bit = (alpha * dot >= thr)
  uint32_t* out_bits;
  const float* thr;  // [O] or null (= 0)
  int Nimg, Ho, oHp, oWp, oCw, opad;
  int P;  // N * Ho * Wo
  int O, HoWo, Wo, Hp, Wpp, Cw, stride;
  int nblocks, nchunks;  // blocks of 32 pixels in all; waves they are dealt out to (evenly)
  int blk_q, blk_r;      // nblocks / nchunks and nblocks % nchunks
  int x4;                // 1: K-words 2 q, 2 q + 1 are 16 consecutive, 16-byte aligned bytes of the image; 2: 4 q .. 4 q + 3 are 32
  FastDiv div_howo, div_wo;
  int off[kMaxWsWords];  // word offset of K-word j relative to the pixel base
};

__device__ __forceinline__ v8i widen(v4i e) {
  v8i x;
#pragma unroll
  for (int d = 0; d < 4; ++d) x[d] = e[d];
#pragma unroll
  for (int d = 4; d < 8; ++d) x[d] = 0;
  return x;
}

// The four bit planes of a dword as the four operand dwords of an MFMA step (nibble i of dword
// d = bit 4 i + d).  The pixel side leaves planes 0 to 2 where they stand in their nibbles
// (E2M1 codes 1, 2, 4 = 0.5, 1, 2) and shifts only the plane under the nibble's sign bit: five
// VALU instructions instead of seven, in a kernel whose VALU work outweighs its MFMA time.  The
// filter side, expanded once per workgroup, carries the reciprocal magnitudes (2, 1, 0.5, 2)
// with the sign of the filter value (bit set: +, bit clear: -, the nibble's sign bit being
// the inverted filter bit), so that a set pixel bit contributes +1 or -1 and a clear one nothing.
__device__ __forceinline__ v4i expand_pixel(uint32_t w) {
  v4i e;
  e[0] = (int)(w & 0x11111111u);
  e[1] = (int)(w & 0x22222222u);
  e[2] = (int)(w & 0x44444444u);
  e[3] = (int)((w >> 3) & 0x11111111u);
  return e;
}
__device__ __forceinline__ v4i expand_filter(uint32_t w) {
  const uint32_t nw = ~w;
  v4i e;
  e[0] = (int)(((nw << 3) & 0x88888888u) | 0x44444444u);
  e[1] = (int)(((nw << 2) & 0x88888888u) | 0x22222222u);
  e[2] = (int)(((nw << 1) & 0x88888888u) | 0x11111111u);
  e[3] = (int)((nw & 0x88888888u) | 0x44444444u);
  return e;
}

// Where lane (r, hh) finds the patch of pixel r of a block, and where the block's results go:
// 32-bit offsets from wave-uniform bases (the launcher takes only problems whose packed image and
// output stay below 4 GiB), so that loads and stores use the scalar-base + lane-offset form and
// need one 32-bit add each instead of 64-bit address arithmetic.
struct PixelBlock {
  uint32_t xoff;   // byte offset of the pixel's patch (tap (0, 0), channel word 0) in the packed image
  uint32_t obase;  // element index of (image, filter 0, pixel) in the output
  uint32_t bword;  // packed-bit output: index of the pixel's first word
  int valid;
};

// Products of a wave-uniform factor and a per-lane factor that both stay below 2^24 (the
// launcher checks) on the 24-bit multiplier: a full 32-bit product takes the vector ALU four
// times as long, and every wave of the launch runs this at the same moment, ahead of its first
// load.  (Written out: the compiler proves the range of few of these factors and falls back
// to the full product for the rest.)
__device__ __forceinline__ uint32_t mul24(uint32_t uniform, uint32_t lane) {
  uint32_t r;
  asm("v_mul_u32_u24 %0, %1, %2" : "=v"(r) : "s"(uniform), "v"(lane));
  return r;
}
__device__ __forceinline__ uint32_t mad24(uint32_t uniform, uint32_t lane, uint32_t add) {
  uint32_t r;
  asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(r) : "s"(uniform), "v"(lane), "v"(add));
  return r;
}

__device__ __forceinline__ PixelBlock locate(const WsParams& p, int b, int r) {
  PixelBlock pb;
  const int n = b * 32 + r;
  const int nc = min(n, p.P - 1);  // lanes past the last pixel repeat it and store nothing
  const uint32_t img = fast_div((uint32_t)nc, p.div_howo);
  const uint32_t rem = (uint32_t)nc - mul24((uint32_t)p.HoWo, img);
  const uint32_t ho = fast_div(rem, p.div_wo);
  const uint32_t wo = rem - mul24((uint32_t)p.Wo, ho);
  const uint32_t row = mad24((uint32_t)p.Hp, img, mul24((uint32_t)p.stride, ho));  // row of the padded image stack
  const uint32_t row_bytes = (uint32_t)(p.Wpp * p.Cw) * 8u, step_bytes = (uint32_t)(p.stride * p.Cw) * 8u;  // (wave-uniform)
  pb.xoff = mad24(row_bytes, row, mul24(step_bytes, wo));
  pb.obase = img * (uint32_t)(p.O * p.HoWo) + rem;
  const uint32_t orow = mad24((uint32_t)p.oHp, img, ho + (uint32_t)p.opad);
  pb.bword = mad24((uint32_t)p.oWp, orow, wo + (uint32_t)p.opad) * (uint32_t)p.oCw;
  pb.valid = n < p.P;
  return pb;
}

// LDS.  Filters: row i of the workgroup's block holds its 8 * KW expanded dwords (for word j
// and half h the four dwords of expand_filter(half) at 8 j + 4 h + d), the float
// K - 2 * popcount and alpha; the row stride of 8 * KW + 4 dwords (4, 12 or 20 mod 32) lets
// eight lanes read eight different bank groups with one 16-byte read each.
// Pixels need no LDS: the words are fetched with neighbouring lanes on neighbouring addresses
// (lane (r, hh) takes word 2i + hh of pixel r; a load in which every lane gathers its own
// pixel's words costs the memory pipeline one access per lane) and reach the MFMA's order
// (dword h of every word of pixel r) by a swap between the half-waves, see `transpose`.
template <int KW>
struct Lds {
  static constexpr int kFilterStride = 8 * KW + 4;  // dwords
};

#ifdef BMX_WS_STAMPS
// Profiling builds only: per-wave shader-clock stamps at the phase boundaries of the kernel.
}  // namespace
unsigned long long* ws_stamps = nullptr;
namespace {
#define WS_STAMP(k) do { if (stamps && lane == 0) stamps[(size_t)((blockIdx.y * gridDim.x + blockIdx.x) * (blockDim.x >> 6) + wave) * 16 + (k)] = __builtin_readcyclecounter(); } while (0)
#define WS_STAMP_ARG , unsigned long long* stamps
constexpr int kWs36Waves = 2;  // (the stamps need registers of their own)
// (the constant 100 MHz counter, which all parts of the chip share: for times between waves)
#define WS_REALTIME(k) do { if (stamps && lane == 0) stamps[(size_t)((blockIdx.y * gridDim.x + blockIdx.x) * (blockDim.x >> 6) + wave) * 16 + (k)] = __builtin_amdgcn_s_memrealtime(); } while (0)
#else
#define WS_STAMP(k) do { } while (0)
#define WS_REALTIME(k) do { } while (0)
#define WS_STAMP_ARG
constexpr int kWs36Waves = 3;  // waves per SIMD at 36 words, 16-byte pixel loads, fp32 or int32 results
#endif

// WPS: waves per SIMD the register allocation is held to.
// BITS: the result leaves as packed sign bits (see WsParams::out_bits); the workgroups also
// write the constant halo words of the output image.

// X4: the pixel words are fetched 16 bytes at a time (1: an even number of channel words, so that
// K-words 2 q and 2 q + 1 are neighbours in the image and 16-byte aligned; 2: a multiple of four
// channel words, so that K-words 4 q .. 4 q + 3 are 32 consecutive bytes and the two half-waves'
// addresses differ by 16 in every load: a uniform base per load and one lane offset for all).
// ONE: every wave has exactly one block (the launcher's choice when the blocks are dealt out
// one per wave and there are two or more waves per SIMD, and at 36 words also when that takes
// four waves per SIMD instead of three): nothing is fetched ahead and no next block located,
// one accumulator chain (the SIMD's other waves fill the matrix pipe while a wave waits for its
// own last MFMA), a scalar base per output row; the wave lives in under 100 registers.
// NW: waves per workgroup (4, or 8 with WPS even): twice the waves share one copy of the filter
// block, so that each expands half as much of it and a CU holds half as many copies.  Worth
// 0.5 us where four waves per SIMD contend for the vector ALU over 36 words (64 x 256 x 14 x 14,
// 256 filters: 8.5 -> 8.0 us), nothing at 9 words, and sixteen waves leave CUs empty there (8.7).
template <int KW, int TM, int WPS, bool BITS, int X4, bool ONE = false, int NW = 4>
__global__ void __launch_bounds__(64 * NW, WPS * 4 / NW)
conv_mfma_ws_kernel(const WsParams p WS_STAMP_ARG) {
  static_assert(NW == 4 || (NW == 8 && WPS % 2 == 0), "whole workgroups per CU");
  constexpr int kThreads = 64 * NW;
  static_assert((!X4 || KW % 2 == 0) && (X4 != 2 || KW % 4 == 0), "pairs of words, or fours");
  // load instructions per block: two words per pixel each, or four
  constexpr int NI = X4 ? (KW + 3) / 4 : (KW + 1) / 2;
  typedef typename std::conditional<X4 != 0, v4u, uint64_t>::type Staged;
  constexpr int FS = Lds<KW>::kFilterStride;
  __shared__ __attribute__((aligned(16))) uint32_t filt[32 * TM * FS];
  // The arguments span six or seven 64-byte lines that no cache holds when the kernel starts,
  // and the compiler fetches them in groups of first use, one memory round trip per group.
  // Fields at most 64 bytes apart, named in one statement here, bring all lines in with the
  // first group; the groups that follow hit the scalar cache.
  static_assert(offsetof(WsParams, Nimg) <= 64 && offsetof(WsParams, blk_q) - offsetof(WsParams, Nimg) <= 64 &&
                    offsetof(WsParams, off) + 7 * 4 - offsetof(WsParams, blk_q) <= 64 &&
                    sizeof(WsParams) - (offsetof(WsParams, off) + 39 * 4) <= 64 && kMaxWsWords > 39,
                "a named field in every 64 bytes");
  asm volatile("" ::"s"(p.Xp), "s"(p.Nimg), "s"(p.blk_q), "s"(p.off[7]), "s"(p.off[23]), "s"(p.off[39]));
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 31, h = lane >> 5;
  const int m0 = blockIdx.y * (32 * TM);
  const int chunk = blockIdx.x * NW + wave;
  // the blocks are dealt out evenly: chunk c takes blk_q of them, the first blk_r chunks one more
  // (no division here: this runs before the wave's first load)
  const int cc = min(chunk, p.nchunks);
  const int b0 = cc * p.blk_q + min(cc, p.blk_r);
  const int b1 = cc < p.nchunks ? b0 + p.blk_q + (cc < p.blk_r ? 1 : 0) : b0;
  WS_STAMP(0);
  WS_REALTIME(4);

  // words 2i + h of the pixel's patch, i = 0 .. NI-1 (the odd KW's last one only for h = 0);
  // X4: words 4i + 2h and 4i + 2h + 1 in one load
  auto fetch = [&](const PixelBlock& pb, Staged (&st)[NI]) {
    const char* const xbytes = (const char*)p.Xp;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      if constexpr (X4 == 2) {
        st[i] = *(const v4u*)((xbytes + (size_t)((uint32_t)p.off[4 * i] * 8u)) + (size_t)(pb.xoff + 16u * (uint32_t)h));
      } else if constexpr (X4 == 1) {
        const bool there = 4 * i + 2 < KW || h == 0;
        const uint32_t off = (uint32_t)(h ? p.off[4 * i + 2 < KW ? 4 * i + 2 : 0] : p.off[4 * i]) * 8u;
        st[i] = there ? *(const v4u*)(xbytes + (pb.xoff + off)) : v4u{0u, 0u, 0u, 0u};
      } else {
        const uint32_t off = (uint32_t)(h ? p.off[2 * i + 1 < KW ? 2 * i + 1 : 0] : p.off[2 * i]) * 8u;
        st[i] = (2 * i + 1 < KW || h == 0) ? *(const uint64_t*)(xbytes + (pb.xoff + off)) : 0;
      }
    }
  };
  // staged words -> dword h of every word of pixel r.  Lane (r, 0) holds word 2i and lane (r, 1)
  // word 2i + 1, each as (lo, hi): swapping the upper half-wave of the lo registers with the
  // lower half-wave of the hi registers (v_permlane32_swap, one instruction) leaves dword h of
  // word 2i in the first and dword h of word 2i + 1 in the second.  (X4: lane (r, 0) holds words
  // 4i and 4i + 1, lane (r, 1) words 4i + 2 and 4i + 3; the same swap on each of the two.)
  auto transpose = [&](const Staged (&st)[NI], uint32_t (&raw)[KW]) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      if constexpr (X4) {
        const v2u t = __builtin_amdgcn_permlane32_swap(st[i][0], st[i][1], false, false);
        const v2u u = __builtin_amdgcn_permlane32_swap(st[i][2], st[i][3], false, false);
        raw[4 * i] = t[0];
        raw[4 * i + 1] = u[0];
        if (4 * i + 2 < KW) {
          raw[4 * i + 2] = t[1];
          raw[4 * i + 3] = u[1];
        }
      } else {
        const v2u t = __builtin_amdgcn_permlane32_swap((uint32_t)st[i], (uint32_t)(st[i] >> 32), false, false);
        raw[2 * i] = t[0];
        if (2 * i + 1 < KW) raw[2 * i + 1] = t[1];
      }
    }
  };

  // ---- the workgroup's filters: neighbouring threads on neighbouring words; all of a thread's
  // loads are issued before the first is written to LDS (one after the other, every load
  // would cost a full memory round trip: 6 of 9 us at K = 36 words)
  // one unit = one 64-bit word of a filter's bits, expanded on the way: 8 bytes read, the two
  // halves' four planes (32 bytes) written
  constexpr int kUnits = 32 * TM * KW;
  constexpr int kCopies = (kUnits + kThreads - 1) / kThreads;
  uint64_t buf[kCopies];
  const uint32_t ld_bytes = (uint32_t)p.ld_dw * 4u;
#pragma unroll
  for (int t = 0; t < kCopies; ++t) {
    const int c = min((int)threadIdx.x + kThreads * t, kUnits - 1);
    const uint32_t row = (uint32_t)c / KW, j = (uint32_t)c - mul24(KW, row);
    // rows past the last filter repeat it; their results are never stored
    // (a 32-bit byte offset from the uniform base: no 64-bit address arithmetic per load)
    const uint32_t frow = (uint32_t)min(m0 + (int)row, p.O - 1);
    buf[t] = *(const uint64_t*)((const char*)p.Wp + (size_t)mad24(ld_bytes, frow, 8u * j));
  }
  float myc0 = 0.0f, myalpha = 1.0f, mythr = 0.0f;  // thread t < 32 * TM carries the constants of row t
  if ((int)threadIdx.x < 32 * TM) {
    const uint32_t m = (uint32_t)min(m0 + (int)threadIdx.x, p.O - 1);
    myc0 = *(const float*)((const char*)p.Wp + (size_t)(mul24(ld_bytes, m) + (uint32_t)p.c0_dw * 4u));
    if (p.alpha) myalpha = *(const float*)((const char*)p.alpha + (size_t)(m * 4u));
    if (BITS && p.thr) mythr = *(const float*)((const char*)p.thr + (size_t)(m * 4u));
  }
  // the first block's pixel words are requested right behind the filter words, which the
  // whole workgroup waits for at its barrier (waves of the last workgroup that have no block
  // fetch block 0 and drop it)
  PixelBlock cur = locate(p, b0 < b1 ? b0 : 0, r);
  Staged st[NI];
  fetch(cur, st);
  WS_STAMP(1);

  // (behind the first fetch, so that its index arithmetic runs under the loads)
  if (BITS && p.opad > 0 && (m0 & 63) == 0) {
    // halo of the output image, word m0 / 64 of every halo pixel: every real channel +1 (the
    // sign of the next layer's zero padding), missing channels 0; spread over the workgroups of
    // this filter tile (left to one of them, its few thousand index computations set the
    // duration of the whole launch)
    const int cw = m0 >> 6;
    const uint64_t ones = (cw == p.oCw - 1 && (p.O & 63)) ? (((uint64_t)1 << (p.O & 63)) - 1) : ~(uint64_t)0;
    const int nh = p.oHp * p.oWp - p.HoWo;
    uint64_t* ob = (uint64_t*)p.out_bits;
    for (int i = blockIdx.x * kThreads + threadIdx.x; i < nh * p.Nimg; i += gridDim.x * kThreads) {
      const int n = i / nh, k = i - n * nh;
      int hh, ww;
      if (k < 2 * p.opad * p.oWp) {  // rows above and below
        hh = k / p.oWp;
        ww = k - hh * p.oWp;
        if (hh >= p.opad) hh += p.Ho;
      } else {  // left and right of the interior rows
        const int j = k - 2 * p.opad * p.oWp;
        const int rr = j / (2 * p.opad), c = j - rr * (2 * p.opad);
        hh = p.opad + rr;
        ww = c < p.opad ? c : p.Wo + c;
      }
      ob[(((int64_t)n * p.oHp + hh) * p.oWp + ww) * p.oCw + cw] = ones;
    }
  }

  {
#pragma unroll
    for (int t = 0; t < kCopies; ++t) {
      const int c = (int)threadIdx.x + kThreads * t;
      // word j of row c / KW at dword row * FS + 8 j = 8 c + 4 row, as FS = 8 KW + 4
      static_assert(FS == 8 * KW + 4, "the index below");
      const int at = 8 * c + 4 * (c / KW);
      if (c < kUnits) {
        *(v4i_alias*)(filt + at) = expand_filter((uint32_t)buf[t]);
        *(v4i_alias*)(filt + at + 4) = expand_filter((uint32_t)(buf[t] >> 32));
      }
    }
    if ((int)threadIdx.x < 32 * TM) {
      filt[(int)threadIdx.x * FS + 8 * KW] = __float_as_uint(myc0);
      filt[(int)threadIdx.x * FS + 8 * KW + 1] = __float_as_uint(myalpha);
      if (BITS) filt[(int)threadIdx.x * FS + 8 * KW + 2] = __float_as_uint(mythr);
    }
  }
  WS_STAMP(2);
  __syncthreads();
  WS_STAMP(3);
  if (b0 >= b1) return;

  // ---- blocks of 32 output pixels
  for (int b = b0; b < b1; ++b) {
    uint32_t raw[KW];
    transpose(st, raw);
    // the next block's words are requested before this block is multiplied (after the wave's
    // last block there is nothing to request)
    PixelBlock nxt = cur;
    if constexpr (!ONE) {
      nxt = locate(p, min(b + 1, b1 - 1), r);
      if (b + 1 < b1) fetch(nxt, st);
    }
    // (the filter reads below are the same in every trip: an opaque copy of their base keeps
    // the compiler from hoisting all of them out of the loop and into registers for good)
    // (counted in 16-byte pieces from the aligned base, so that the read is one ds_read_b128:
    // split into dword pairs, the lanes of eight rows would meet on four banks)
    int fbase = r * (FS / 4) + h;
    asm volatile("" : "+v"(fbase));
    if (b == b0) WS_STAMP(10);
    // Two accumulator chains per filter block, steps alternating between them and added at the
    // end: an MFMA that adds onto the result of the one before it can only start when that one
    // has finished, twice the time it takes to issue.  The filter operands are read a group of
    // steps ahead: read where they are used, every pair of MFMAs would wait out an LDS round trip.
    // (with two filter blocks per wave their two chains are independent already, and registers
    // are short: one chain each, operands two steps ahead; the one-block form runs with two or
    // more waves per SIMD, whose chains interleave: one chain, and no sixteen additions)
    constexpr int CH = (TM == 1 && !ONE) ? 2 : 1;
    constexpr int G = (KW > 36 || TM == 2) ? 2 : 4, NG = (KW + G - 1) / G;
    v16f acc[TM][CH];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int c = 0; c < CH; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][c][e] = 0.0f;
    v4i abuf[2][G][TM];
    auto load_group = [&](int g, v4i (&dst)[G][TM]) {
#pragma unroll
      for (int t = 0; t < G; ++t)
#pragma unroll
        for (int i = 0; i < TM; ++i)
          if (g * G + t < KW) dst[t][i] = ((const v4i_alias*)filt)[fbase + 8 * i * FS + 2 * (g * G + t)];
    };
    load_group(0, abuf[0]);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      if (g + 1 < NG) load_group(g + 1, abuf[(g + 1) & 1]);
#pragma unroll
      for (int t = 0; t < G; ++t) {
        const int j = g * G + t;
        if (j < KW) {
          const v8i eb = widen(expand_pixel(raw[j]));
#pragma unroll
          for (int i = 0; i < TM; ++i)
            acc[i][j % CH] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(widen(abuf[g & 1][t][i]), eb, acc[i][j % CH], 4, 4,
                                                                            0, 127, 0, 127);  // (block scales of 1)
        }
      }
      // keep the operands of the groups that follow behind these MFMAs: gathered at the top of
      // the block (the scheduler's preference) they would hold 8 * KW registers at once
      __builtin_amdgcn_sched_barrier(0);
    }
    if (b == b0) WS_STAMP(8);
    if constexpr (CH == 2) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][0][e] += acc[i][1][e];  // exact: whole numbers below 2^24
    }
    if (b == b0) WS_STAMP(9);
    // out = alpha * ((K - 2 pc(filter)) + 2 * sum): exact integers in fp32 up to the single
    // rounding of the alpha product.  (The row constants of all result registers in one batch
    // of LDS reads: read one by one inside the store loop, every value would pay a full LDS
    // round trip.)
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      float c0[16], al[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int mi = 32 * i + 8 * (v / 4) + 4 * h + (v % 4);  // row of result register v
        c0[v] = __uint_as_float(filt[mi * FS + 8 * KW]);
        al[v] = __uint_as_float(filt[mi * FS + 8 * KW + 1]);
      }
      if constexpr (BITS) {
        // bit o of the pixel's word: the IEEE compare of the fp32 product, as packing the fp32
        // result would see it; the lane pair (r, 0), (r, 1) holds the 32 filters between them
        uint32_t mask = 0;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int mi = 8 * (v / 4) + 4 * h + (v % 4);
          const float th = __uint_as_float(filt[(32 * i + mi) * FS + 8 * KW + 2]);
          const float t = fmaf(2.0f, acc[i][0][v], c0[v]);
          if (al[v] * t >= th && m0 + 32 * i + mi < p.O) mask |= 1u << mi;
        }
        mask |= (uint32_t)__shfl_xor((int)mask, 32);
        const int mb = m0 + 32 * i;
        if (h == 0 && cur.valid && mb < p.O) {
          uint32_t* dst = p.out_bits + 2 * (cur.bword + (mb >> 6)) + ((mb >> 5) & 1);
          dst[0] = mask;
          if ((mb & 32) == 0 && mb + 32 >= p.O) dst[1] = 0;  // nobody else owns the upper half
        }
      } else {
        // Register v goes to row m0 + 32 i + 8 (v / 4) + 4 h + v % 4, pixel r: one wave-uniform
        // base for the whole output and a 32-bit lane offset per register (the block's offset
        // plus a multiple of the row pitch).  A block wholly inside the output (the usual case)
        // stores without bounds tests.
        const uint32_t pitch = (uint32_t)p.HoWo * 4u;
        const uint32_t lane_off = cur.obase * 4u + (uint32_t)(m0 + 32 * i + 4 * h) * pitch;
        const bool inside = b * 32 + 32 <= p.P && m0 + 32 * TM <= p.O;
        auto put = [&](auto inside_tag, auto int_tag) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int mi = 8 * (v / 4) + (v % 4);
            // (ONE: the row's share of the address goes into the uniform base, on the scalar ALU,
            // and all sixteen stores share one lane offset; with several blocks per wave the
            // compiler would keep sixteen such bases across the block loop and run out of SGPRs)
            const uint32_t off = ONE ? lane_off : lane_off + (uint32_t)mi * pitch;
            const size_t row_bytes = ONE ? (size_t)mi * pitch : 0;
            const float t = fmaf(2.0f, acc[i][0][v], c0[v]);
            if (decltype(inside_tag)::value || (cur.valid && m0 + 32 * i + mi + 4 * h < p.O)) {
              // (written out: the compiler builds a 64-bit vector address for a non-temporal
              // store even from a uniform base and a 32-bit offset)
              if constexpr (decltype(int_tag)::value) {
                const int iv = (int)t;
                asm volatile("global_store_dword %0, %1, %2 nt" ::"v"(off), "v"(iv), "s"((const char*)p.out_i32 + row_bytes) : "memory");
              } else {
                const float fv = al[v] * t;
                asm volatile("global_store_dword %0, %1, %2 nt" ::"v"(off), "v"(fv), "s"((const char*)p.out_f32 + row_bytes) : "memory");
              }
            }
          }
        };
        if (p.out_i32) {
          if (inside) put(std::true_type{}, std::true_type{});
          else put(std::false_type{}, std::true_type{});
        } else {
          if (inside) put(std::true_type{}, std::false_type{});
          else put(std::false_type{}, std::false_type{});
        }
      }
    }
    if constexpr (ONE) break;
    cur = nxt;
  }
  WS_STAMP(6);
#ifdef BMX_WS_STAMPS
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  WS_STAMP(7);
  WS_REALTIME(5);
#endif
}

template <int KW, int TM, int WPS, bool BITS, int X4, bool ONE = false, int NW = 4>
void launch_ws_form(const WsParams& p, int m_tiles, hipStream_t s) {
  const int chunks = p.nchunks;
  note_kernel("conv_mfma_ws_kernel<%d,%d,%d,%s%s%s> grid %d x %d x %d", KW, TM, WPS, BITS ? "true" : "false",
              X4 == 2 ? ",x4 runs" : X4 ? ",x4" : "", ONE ? ",one block" : "", (int)ceil_div(chunks, NW), m_tiles, 64 * NW);
#ifdef BMX_WS_STAMPS
  hipLaunchKernelGGL((conv_mfma_ws_kernel<KW, TM, WPS, BITS, X4, ONE, NW>), dim3((unsigned)ceil_div(chunks, NW), (unsigned)m_tiles),
                     dim3(64 * NW), 0, s, p, ws_stamps);
#else
  hipLaunchKernelGGL((conv_mfma_ws_kernel<KW, TM, WPS, BITS, X4, ONE, NW>), dim3((unsigned)ceil_div(chunks, NW), (unsigned)m_tiles),
                     dim3(64 * NW), 0, s, p);
#endif
}

// WPS_X4: waves per SIMD of the form with 16-byte pixel loads, which needs fewer registers.
template <int KW, int TM, int WPS, bool BITS = false, int WPS_X4 = WPS>
void launch_ws(const WsParams& p, int m_tiles, hipStream_t s) {
  // 16-byte pixel loads where the word count can come from an even number of channel words
  if constexpr (KW == 18 || KW == 36 || KW == 50) {
    if constexpr (KW == 36) {
      if (p.x4 == 2) return launch_ws_form<KW, TM, WPS_X4, BITS, 2>(p, m_tiles, s);
    }
    if (p.x4) return launch_ws_form<KW, TM, WPS_X4, BITS, 1>(p, m_tiles, s);
  }
  launch_ws_form<KW, TM, WPS, BITS, 0>(p, m_tiles, s);
}

}  // namespace

bool conv_mfma_ws_takes(int Nimg, int C, int H, int W, int O, int KH, int KW, int stride, int pad,
                        int out_pad) {
  const int Ho = (H + 2 * pad - KH) / stride + 1;
  const int Wo = (W + 2 * pad - KW) / stride + 1;
  const int Cw = (int)words_for(C);
  const int kwords = KH * KW * Cw;
  if (!conv_weight_short_k(kwords)) return false;
  const int64_t P = (int64_t)Nimg * Ho * Wo;
  if (P >= ((int64_t)1 << 31) || (int64_t)C * KH * KW >= ((int64_t)1 << 22)) return false;
  if ((int64_t)Nimg * (Ho + 2 * out_pad) * (Wo + 2 * out_pad) >= ((int64_t)1 << 31)) return false;
  if ((int64_t)(KH * (W + 2 * pad) + KW) * Cw >= ((int64_t)1 << 30)) return false;
  // packed image, output and packed-bit output are addressed with 32-bit byte offsets
  if ((int64_t)Nimg * (H + 2 * pad) * (W + 2 * pad) * Cw * 8 >= ((int64_t)1 << 32)) return false;
  if (((int64_t)Nimg * O + 64) * Ho * Wo * 4 >= ((int64_t)1 << 32)) return false;
  // the packed filters as well, and the factors of the kernel's 24-bit products
  if ((int64_t)(O + 64) * 2 * conv_weight_row_words(kwords) * 4 >= ((int64_t)1 << 32)) return false;
  const int64_t lim24 = (int64_t)1 << 24;
  if ((int64_t)Nimg * (H + 2 * pad) >= lim24 || (int64_t)(W + 2 * pad) * Cw * 8 >= lim24 || (int64_t)stride * Cw * 8 >= lim24 ||
      (int64_t)Ho * Wo >= lim24 || (int64_t)Nimg * (Ho + 2 * out_pad) >= lim24 || (int64_t)Wo + 2 * out_pad >= lim24 || O >= lim24)
    return false;
  if ((int64_t)Nimg * (Ho + 2 * out_pad) * (Wo + 2 * out_pad) * words_for(O) * 8 >= ((int64_t)1 << 32)) return false;
  return ceil_div(O, 32) <= 65535;
}

bool launch_conv_mfma_ws(const uint64_t* Xp, int Nimg, int C, int H, int W, const uint64_t* Wp, int O,
                         int KH, int KW, int stride, int pad, const float* alpha, int32_t* out_i32,
                         float* out_f32, uint64_t* out_bits, const float* thr, int out_pad, hipStream_t s,
                         hipError_t* err) {
  if (!conv_mfma_ws_takes(Nimg, C, H, W, O, KH, KW, stride, pad, out_bits ? out_pad : 0) ||
      ((uintptr_t)Wp & 15))
    return false;
  const int Ho = (H + 2 * pad - KH) / stride + 1;
  const int Wo = (W + 2 * pad - KW) / stride + 1;
  const int Cw = (int)words_for(C);
  const int kwords = KH * KW * Cw;
  const int64_t P = (int64_t)Nimg * Ho * Wo;
  WsParams p;
  p.Xp = Xp;
  p.Wp = (const uint32_t*)Wp;
  p.ld_dw = 2 * (int)conv_weight_row_words(kwords);
  p.c0_dw = 2 * (int)conv_weight_bits_words(kwords);
  p.alpha = alpha;
  p.out_i32 = out_i32;
  p.out_f32 = out_f32;
  p.out_bits = (uint32_t*)out_bits;
  p.thr = thr;
  p.Nimg = Nimg;
  p.Ho = Ho;
  p.opad = out_pad;
  p.oHp = Ho + 2 * out_pad;
  p.oWp = Wo + 2 * out_pad;
  p.oCw = (int)words_for(O);
  p.P = (int)P;
  p.O = O;
  p.HoWo = Ho * Wo;
  p.Wo = Wo;
  p.Hp = H + 2 * pad;
  p.Wpp = W + 2 * pad;
  p.Cw = Cw;
  p.stride = stride;
  p.div_howo = make_fast_div((uint32_t)(Ho * Wo));
  p.div_wo = make_fast_div((uint32_t)Wo);
  for (int j = 0; j < kMaxWsWords; ++j) p.off[j] = 0;
  for (int kh = 0; kh < KH; ++kh)
    for (int kw = 0; kw < KW; ++kw)
      for (int cw = 0; cw < Cw; ++cw) p.off[(kh * KW + kw) * Cw + cw] = (kh * p.Wpp + kw) * Cw + cw;
  p.nblocks = (int)ceil_div(P, 32);
  // (64 filters per workgroup, two accumulator sets sharing every expanded pixel word, is kept
  // for measurements only: it lost to 32 everywhere, 8.0 against 7.2 us on 16 x 64 x 56 x 56)
  // (also tried at 36 words.  As written the compiler runs the first filter block's whole chain
  // before the second's and parks the second's operands in scratch, 185 registers' worth; with
  // the two accumulators tied together after every group of steps it needs 167 registers and
  // none in scratch, and then takes 8.9 us against 8.6 on 64 x 256 x 14 x 14 with 256 filters: the busiest SIMD
  // has 144 MFMAs either way, and the workgroup's filter copy is twice as long; the same again in
  // the form with one block per wave: 8.9 against 8.1 us)
  const int TM = (kwords == 9 && O > 32 && gemm_mfma_tile == 2 && !out_bits) ? 2 : 1;
  const int m_tiles = (int)ceil_div(O, 32 * TM);
  // Waves: one per block while all of them are resident at once (workgroups per CU as the
  // registers allow: 4 at 9 words, 3 up to 27 and, with 16-byte pixel loads and fp32 or int32
  // results, at 36, else 2); beyond that, as many waves as are resident in one round, the
  // blocks dealt out evenly: every workgroup copies its filters once and no CU is left with a
  // second round of a few workgroups.
  p.x4 = ((Cw & 1) == 0 && ((uintptr_t)Xp & 15) == 0 && conv_ws_x4 != 1) ? 1 : 0;
  if (p.x4 && (Cw & 3) == 0 && conv_ws_x4 != 2) p.x4 = 2;
  const int per_simd = kwords == 9 ? 4 : kwords <= 27 ? 3 : (kwords == 36 && p.x4 && !out_bits) ? kWs36Waves : 2;
  const int resident_waves = 256 * 4 * per_simd;
  p.nchunks = (int)std::min<int64_t>(p.nblocks, std::max(1, resident_waves / m_tiles));
  // At 36 words over four channel words: when a wave per block fits at four waves per SIMD but
  // not at three, the form that holds one block in under 100 registers (in workgroups of eight
  // waves); no wave is then left with a second block to run alone after the others have gone.
  const bool one36 = kwords == 36 && p.x4 == 2 && !out_bits && TM == 1 && p.nchunks < p.nblocks &&
                     (int64_t)p.nblocks * m_tiles <= 256 * 4 * 4 && conv_filters_per_wave == 0 && conv_ws_x4 != 3;
  if (one36) p.nchunks = p.nblocks;
  if (conv_filters_per_wave >= 100) p.nchunks = std::min(p.nblocks, conv_filters_per_wave);  // (tuning hook reused: chunks)
  else if (conv_filters_per_wave > 0) p.nchunks = (int)ceil_div(p.nblocks, conv_filters_per_wave);  // (or blocks per wave)
  p.blk_q = p.nblocks / p.nchunks;
  p.blk_r = p.nblocks % p.nchunks;
  if (out_bits) {
    if (kwords == 9 && p.nchunks == p.nblocks && (int64_t)p.nblocks * m_tiles >= 2048 && conv_ws_x4 != 3)
      launch_ws_form<9, 1, 4, true, 0, true>(p, m_tiles, s);
    else if (kwords == 9) launch_ws<9, 1, 4, true>(p, m_tiles, s);
    else if (kwords == 18) launch_ws<18, 1, 3, true>(p, m_tiles, s);
    else if (kwords == 25) launch_ws<25, 1, 3, true>(p, m_tiles, s);
    else if (kwords == 27) launch_ws<27, 1, 3, true>(p, m_tiles, s);
    else if (kwords == 49) launch_ws<49, 1, 2, true>(p, m_tiles, s);
    else if (kwords == 50) launch_ws<50, 1, 2, true>(p, m_tiles, s);
    else launch_ws<36, 1, 2, true>(p, m_tiles, s);
  } else if (kwords == 9) {
    if (TM == 2) launch_ws<9, 2, 2>(p, m_tiles, s);
    // (a wave per block: the form that fetches nothing ahead and keeps one accumulator chain)
    // (from two waves per SIMD on: a wave alone on its SIMD is better off with two chains)
    else if (p.nchunks == p.nblocks && (int64_t)p.nblocks * m_tiles >= 2048 && conv_ws_x4 != 3)
      launch_ws_form<9, 1, 4, false, 0, true>(p, m_tiles, s);
    else launch_ws<9, 1, 4>(p, m_tiles, s);
  } else if (kwords == 18) {
    launch_ws<18, 1, 3>(p, m_tiles, s);
  } else if (kwords == 25) {
    launch_ws<25, 1, 3>(p, m_tiles, s);
  } else if (kwords == 27) {
    launch_ws<27, 1, 3>(p, m_tiles, s);
  } else if (kwords == 49) {
    launch_ws<49, 1, 2>(p, m_tiles, s);
  } else if (kwords == 50) {
    launch_ws<50, 1, 2>(p, m_tiles, s);
  } else if (one36) {  // (with a wave per block anyway the other form is as fast: 5.2 against 5.3 us at stride 2)
    launch_ws_form<36, 1, 4, false, 2, true, 8>(p, m_tiles, s);
  } else {
    launch_ws<36, 1, 2, false, kWs36Waves>(p, m_tiles, s);
  }
  *err = hipGetLastError();
  return true;
}

}  // namespace bmx
