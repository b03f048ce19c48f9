// xnor GEMM and bit-plane GEMM on the FP4 matrix cores: 64 x 64 of C per wave, operands staged
// through LDS by the load unit itself, K split over the waves of a workgroup.
// Paper: Sec. 2.2.1 / Sec. 2.2.2 (Eq. 2): C[m][n] = K - 2 * popcount(A[m] xor B[n]); Sec. 2.1
// (Eq. 1) for the k-bit activations of the plane form.
//
// Arithmetic (as in gemm_mfma.hip): with bits a, b in {0, 1},
//     K - 2 * pc(a xor b) = K - 2 * pc(a) - 2 * pc(b) + 4 * sum_k a * b,
// the sum on v_mfma_scale_f32_32x32x64_f8f6f4 with both operands FP4 (E2M1).  A bit stays where
// it stands in its nibble (worth 0.5, 1 or 2 there; the nibble's top bit is shifted down) and
// the block scale of each MFMA brings the product back to 1, so one 32-bit word of bits becomes
// the four 8-nibble operand dwords of four MFMAs with five VALU instructions.  Products and
// fp32 sums are exact integers below 2^24.  The two bit planes of a 2-bit activation are staged
// as separate rows and folded into one operand while being expanded: a nibble then holds the
// 2-bit value itself (E2M1 codes 0 to 3 = 0, 0.5, 1, 1.5; block scale 2).
//
// What bounds this kernel is not the matrix core but everything around it: the VALU work of
// turning bits into nibbles, the loads, and fixed costs of a few-microsecond launch.  Hence:
//   - 2 x 2 blocks of 32 x 32 per wave: an expanded operand block serves two MFMAs, 5 VALU
//     instructions of expansion and 1 of row popcount per MFMA (a 32 x 32 tile needs 12).
//   - Operands travel global memory -> LDS without passing registers (global_load_lds_dwordx4:
//     lane i of the instruction writes LDS bytes [16 i, 16 i + 16) of its destination).  A load
//     covers 16 rows x 64 bytes, 4 lanes per row: whole 64-byte runs, so the memory pipeline
//     works at its coalesced rate, where the MFMA layout (lane = row) costs an access per lane.
//     Which 16-byte piece a lane fetches is permuted (piece = slot xor ((row >> 1) & 3)), so
//     that the MFMA-layout reads, lane (r, h) <- piece 2 g + h of row r, fall on all banks.
//   - A wave owns its staging area and its range of K: no barrier in the main loop.  The words
//     of a 64-byte segment are read into registers, the next segment's loads are issued into
//     the same area once those reads have completed, and the 32 MFMAs of the segment run with
//     those loads in flight.
//   - Skinny problems (the fully connected layers: 256 rows) have too few 64 x 64 tiles to
//     fill the chip, so the S waves of a workgroup split K and add their partial tiles through
//     LDS once: every wave writes its 64 registers, then finishes 1/S of the tile (sum of S
//     partials, the popcount terms, scale, store).  Fat problems run four tiles per workgroup
//     and no split.
//   - Workgroups are numbered so that tiles sharing operand rows sit on one XCD and run back
//     to back (workgroup b runs on XCD b % 8): every XCD gets a contiguous run of tiles, walked
//     in bands of 16 rows of tiles.
//   - The convolution form gathers the B operand (im2col rows) from the halo-padded packed
//     image, 16 bytes per lane, through the same loads.
#include <algorithm>
#include <type_traits>

#include "bmx_internal.h"

namespace bmx {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v4i_alias __attribute__((ext_vector_type(4), may_alias));
typedef __fp16 half2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lds_ptr;

struct Fp4Params {
  const uint64_t* A;  // [M * PL][lda] words (plane pl of row m is row m * PL + pl), tail bits zero
  const uint64_t* B;  // [N][ldb] words
  uint32_t lda_bytes, ldb_bytes;  // row strides, multiples of 16
  int M, N, Kw, Kreal;            // Kw data words per row
  int g_base, g_rem;  // groups of four words (256 bits = the K of four MFMAs) per wave: g_base, the first g_rem waves one more
  int tiles_m, tiles_n, tiles_per_xcd;
  // tile order: bands of `band` rows of tiles (the last band has last_rows), see the kernel
  int band, per_band, last_band, last_rows;
  FastDiv div_per_band, div_band, div_last;
  const float* alpha;     // per column n, or null
  const float* thr;       // packed-bit output: per column threshold of the sign decision, or null (0)
  const int32_t* rowsum;  // plane form: sum_k q[m][k]
  float levels;           // plane form: 2^bits - 1
  int as_count;           // int32 output holds the xnor count (dot + K) / 2
  int32_t* C_i32;
  float* C_f32;
  uint32_t* C_bits;  // packed sign bits, addressed in 32-bit halves of the output words
  int ldc;           // elements per row (C_bits: 64-bit words per row); M * ldc < 2^31
  // Convolution form (Sec. 3.1: M = filters, N = batch * output pixels, K = kh * kw * C): A is the
  // packed filter matrix, B the halo-padded packed image.  Column n is output pixel n (flat over
  // the images); its K words are KH runs of KW * Cw consecutive words, one run per kernel row
  // (the taps of a kernel row are neighbouring pixels, channel words innermost), so with an even
  // Cw every 16-byte piece of the im2col row is 16 consecutive bytes of the image.  alpha is per
  // row m here, and the result goes to NCHW: element (image * M + m) * HoWo + pixel.
  int HoWo, Wo, Hp, Wpp, Cw, stride;
  uint32_t run_pieces, row_bytes, npieces;  // pieces per run; bytes from run to run; pieces per pixel
  FastDiv div_howo, div_wo, div_run;
};

// One nibble plane of four words of bits as the four operand dwords of one MFMA.
//   n = 0: w & 0x11111111 (0.5)   n = 1: w & 0x22222222 (1.0)   n = 2: w & 0x44444444 (2.0)
//   n = 3: (w >> 3) & 0x11111111 (0.5), hi = w >> 3 computed once per word
__device__ __forceinline__ v8i nibble_plane(const uint4& w, const uint4& hi, int n) {
  v8i e;
  if (n == 3) {
    e[0] = (int)(hi.x & 0x11111111u);
    e[1] = (int)(hi.y & 0x11111111u);
    e[2] = (int)(hi.z & 0x11111111u);
    e[3] = (int)(hi.w & 0x11111111u);
  } else {
    const uint32_t m = 0x11111111u << n;
    e[0] = (int)(w.x & m);
    e[1] = (int)(w.y & m);
    e[2] = (int)(w.z & m);
    e[3] = (int)(w.w & m);
  }
  e[4] = e[5] = e[6] = e[7] = 0;
  return e;
}

// Nibble plane n of two bit planes at once: nibble i of a dword = (bit 4 i + n of p1) * 2 + (bit
// 4 i + n of p0), the 2-bit value in the nibble's two low bits.
__device__ __forceinline__ v8i nibble_pair(const uint4& p0, const uint4& p1, int n) {
  const uint32_t a0[4] = {p0.x, p0.y, p0.z, p0.w}, a1[4] = {p1.x, p1.y, p1.z, p1.w};
  v8i e;
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t lo = (a0[d] >> n) & 0x11111111u;
    const uint32_t hi = n == 0 ? (a1[d] & 0x11111111u) << 1 : (a1[d] >> (n - 1)) & 0x22222222u;
    e[d] = (int)(lo | hi);
  }
  e[4] = e[5] = e[6] = e[7] = 0;
  return e;
}

// acc + popcount of four words: four v_bcnt_u32_b32, each adding onto the running count (written
// as a sum of __builtin_popcount the compiler counts from zero and adds with extra instructions)
__device__ __forceinline__ int add_popcount4(int acc, const uint4& w) {
  asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(w.x));
  asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(w.y));
  asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(w.z));
  asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(w.w));
  return acc;
}

// Request segment `seg` (64 bytes of every row of the wave's NB staged blocks) into the staging
// area at dst: per block two loads of 16 rows, lane i of a load writing LDS bytes [16 i, 16 i + 16)
// of its destination.  voff: a lane's byte offset of its piece in segment 0 of its row (CONV: for
// the B blocks, of its pixel's patch; the piece's place inside the patch is found here).
template <int NA, int NB, bool CONV>
__device__ __forceinline__ void issue_segment(const Fp4Params& p, uint4* dst, const uint32_t* voff /* [NB][2] */,
                                              int piece0, int piece1, int seg) {
  const char* abase = (const char*)p.A + (uint32_t)seg * 64u;
  const char* bbase = (const char*)p.B + (CONV ? 0u : (uint32_t)seg * 64u);
  const bool tail = 8 * seg + 8 > p.Kw;  // the row ends inside this segment
  uint32_t boff[2] = {0u, 0u};
  if (CONV) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      // piece c of the im2col row: run c / run_pieces (a kernel row), piece c % run_pieces of it; a
      // piece beyond the row's last is not fetched (the reader zeroes it): its lane repeats the
      // segment's first piece, which always exists
      uint32_t c = 4u * (uint32_t)seg + (uint32_t)(t ? piece1 : piece0);
      if (c >= p.npieces) c = 4u * (uint32_t)seg;
      const uint32_t run = fast_div(c, p.div_run);
      boff[t] = run * p.row_bytes + (c - run * p.run_pieces) * 16u;
    }
  }
#pragma unroll
  for (int b = NB - 1; b >= 0; --b)  // (B first: its rows are the ones that come from far away)
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int pc = t ? piece1 : piece0;
      uint32_t off = voff[2 * b + t];
      if (CONV && b >= NA) off += boff[t];
      // (plain rows) a piece that starts beyond the row's last word: repeat the segment's first
      else if (tail && 8 * seg + 2 * pc >= p.Kw) off -= 16u * pc;
      __builtin_amdgcn_global_load_lds((b < NA ? abase : bbase) + off, (lds_ptr)(dst + b * 128 + t * 64), 16, 0, 0);
    }
}

#ifdef BMX_FP4_STAMPS
// Profiling builds only: per-wave shader-clock stamps at the phase boundaries of the kernel.
}  // namespace
unsigned long long* fp4_stamps = nullptr;
namespace {
#define FP4_STAMP(k) do { if (stamps && lane == 0) stamps[(size_t)(blockIdx.x * (blockDim.x >> 6) + wave) * 8 + (k)] = __builtin_readcyclecounter(); } while (0)
// (without a split, slots 4 and 5 take the constant 100 MHz counter at the loop's ends: with the shader-clock stamps 1 and 3 that gives the clock the loop ran at)
#define FP4_REALTIME(k) do { if (!SPLIT && stamps && lane == 0) stamps[(size_t)(blockIdx.x * (blockDim.x >> 6) + wave) * 8 + (k)] = __builtin_amdgcn_s_memrealtime(); } while (0)
#else
#define FP4_REALTIME(k) do { } while (0)
#define FP4_STAMP(k) do { } while (0)
#endif

// Output kinds of the xnor form (the plane form stores S and / or S / levels as its pointers say).
constexpr int kOutF32 = 0, kOutI32 = 1, kOutBits = 2;

// TM x TN blocks of 32 x 32 per wave; PL bit planes per A row; XNOR: the xnor form (row
// popcounts from the words themselves), else the plane form (row sums given); OUT: what the
// xnor form stores; SPLIT: K split over the S waves of the workgroup (else a tile per wave);
// HALF: the partial tiles of a split cross LDS as fp16 pairs (exact while a wave's sums stay
// at or below 2048, which the launcher checks); CONV: the convolution form (see Fp4Params).
// One instantiation per combination keeps each kernel's code short: the instruction cache
// starts cold at every launch, and a launch lasts a few microseconds.
template <int TM, int TN, int PL, bool XNOR, int OUT, bool SPLIT, bool HALF, bool CONV>
__global__ void __launch_bounds__(512)
gemm_fp4_kernel(const Fp4Params p, const int S_arg
#ifdef BMX_FP4_STAMPS
                , unsigned long long* stamps
#endif
) {
  extern __shared__ uint4 lds[];
  constexpr int NA = TM * PL, NB = NA + TN;  // staged blocks of 32 rows: A's, then B's
  constexpr int kStage = NB * 128;           // uint4 per staged segment: NB blocks x 32 rows x 64 bytes
  constexpr int kGroups = TM * TN * 4;       // a wave's accumulators in units of four registers
  constexpr int kCnt = (TM + TN) * 8;        // uint4 holding a wave's 32 (TM + TN) popcounts
  // LDS per wave: its staging area, overlaid after the main loop of a split by its partial tile
  // + counts.
  constexpr int kPart = HALF ? kGroups * 32 : kGroups * 64;  // uint4 holding a wave's partial tile
  constexpr int kSlot = (!SPLIT || kStage > kPart + kCnt) ? kStage : kPart + kCnt;
  // Everything the wave needs before its first load, named in one statement at the top: the
  // compiler then fetches the kernel arguments in one batch of scalar loads with one wait instead
  // of one memory round trip per group of first uses.
  asm volatile("" ::"s"(p.A), "s"(p.B), "s"(p.lda_bytes), "s"(p.ldb_bytes), "s"(p.M), "s"(p.N), "s"(p.Kw), "s"(p.g_base),
               "s"(p.g_rem), "s"(p.tiles_m), "s"(p.tiles_n), "s"(p.tiles_per_xcd), "s"(p.band), "s"(p.per_band),
               "s"(p.last_band), "s"(p.last_rows), "s"(p.div_per_band.mul), "s"(p.div_per_band.sh1),
               "s"(p.div_per_band.sh2), "s"(p.div_band.mul), "s"(p.div_band.sh1), "s"(p.div_band.sh2),
               "s"(p.div_last.mul), "s"(p.div_last.sh1), "s"(p.div_last.sh2), "s"(S_arg), "s"(p.alpha), "s"(p.thr), "s"(p.rowsum));
  const int S = SPLIT ? S_arg : 1;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane & 31, h = lane >> 5;
  FP4_STAMP(0);
  const int ks = SPLIT ? wave : 0;          // this wave's part of K
  const int tile_in_wg = SPLIT ? 0 : wave;  // without a split every wave has a tile of its own
  const int tiles_per_wg = SPLIT ? 1 : (int)(blockDim.x >> 6);
  // workgroup b sits on XCD b % 8: give every XCD a contiguous run of tiles, rows of C fastest
  const int lin = ((int)(blockIdx.x & 7) * p.tiles_per_xcd + (int)(blockIdx.x >> 3)) * tiles_per_wg + tile_in_wg;
  const bool live = lin < p.tiles_m * p.tiles_n;
  if (!SPLIT && !live) return;  // (no barrier ahead without a split)
  // Within an XCD's run the tiles go band by band: a band is `band` rows of tiles high, and
  // inside it the rows of C run fastest, so the few hundred tiles in flight on an XCD at any time
  // form a block about as wide as high and share their operand rows through its L2.
  int tile_m = 0, tile_n = 0;
  if (live) {  // (divisions by multiply-high with constants from the host: this runs before the first load)
    const int bnd = (int)fast_div((uint32_t)lin, p.div_per_band), within = lin - bnd * p.per_band;
    const bool last = bnd == p.last_band;
    tile_n = (int)fast_div((uint32_t)within, last ? p.div_last : p.div_band);
    tile_m = bnd * p.band + (within - tile_n * (last ? p.last_rows : p.band));
  }
  const int m0 = tile_m * (32 * TM), n0 = tile_n * (32 * TN);

  // ---- this wave's K range in groups of four words.  The first g_rem waves carry one group
  // more: waves w and w + 4 share a SIMD, so with the extras up front the SIMDs stay level (36
  // groups over 8 waves: 5 5 5 5 4 4 4 4, nine per SIMD).
  const int g_lo = ks * p.g_base + min(ks, p.g_rem), g_hi = g_lo + p.g_base + (ks < p.g_rem ? 1 : 0);
  const int seg_lo = g_lo >> 1, seg_hi = (g_hi + 1) >> 1;  // 64-byte segments [seg_lo, seg_hi) of two groups

  // ---- loader: lane i of load t of a block fetches, for local row 16 t + i / 4, the piece
  // (i % 4) xor ((row >> 1) & 3) of the segment; voff = byte offset of that piece in segment 0.
  uint4* const stage = lds + wave * kSlot;
  int piece[2];
  uint32_t voff[NB][2];
#pragma unroll
  for (int t = 0; t < 2; ++t) piece[t] = (lane & 3) ^ (((16 * t + (lane >> 2)) >> 1) & 3);
#pragma unroll
  for (int b = NB - 1; b >= 0; --b)  // (B first: its rows are the ones that come from far away)
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int rl = 16 * t + (lane >> 2);
      if (b < NA) {  // block b = row block b / PL, plane b % PL
        const int m = min(m0 + 32 * (b / PL) + rl, p.M - 1);
        voff[b][t] = (uint32_t)(m * PL + (b % PL)) * p.lda_bytes + 16u * piece[t];
      } else {
        const int n = min(n0 + 32 * (b - NA) + rl, p.N - 1);
        if (CONV) {  // byte offset of the pixel's patch: tap (0, 0), channel word 0
          const uint32_t img = fast_div((uint32_t)n, p.div_howo);
          const uint32_t rem = (uint32_t)n - img * (uint32_t)p.HoWo;
          const uint32_t ho = fast_div(rem, p.div_wo);
          const uint32_t wo = rem - ho * (uint32_t)p.Wo;
          voff[b][t] = (((img * (uint32_t)p.Hp + ho * (uint32_t)p.stride) * (uint32_t)p.Wpp + wo * (uint32_t)p.stride) *
                        (uint32_t)p.Cw) * 8u;
        } else {
          voff[b][t] = (uint32_t)n * p.ldb_bytes + 16u * piece[t];
        }
      }
    }
  // reader: lane (r, h) takes piece 2 g + h of row r for group g of the segment
  int rd[2];
#pragma unroll
  for (int g = 0; g < 2; ++g) rd[g] = (r >> 4) * 64 + (r & 15) * 4 + ((2 * g + h) ^ ((r >> 1) & 3));

  // The epilogue's constants are requested first of all (fetched where they are used, each would
  // put a trip to memory between the main loop and the stores; and ahead of the segments'
  // loads they do not disturb the count of loads in flight that the main loop relies on).  Per column of
  // this lane (column 32 j + r): alpha and the threshold of the sign decision; per row of the
  // tile, row m0 + l in lane l: the row sum of the plane form, alpha of the convolution form.
  static_assert(TM == 2 || (XNOR && !SPLIT && !CONV), "one lane per row of the tile");
  // (plain variables, not arrays: indexed by a run-time j in the reduction below, an array is
  // put into scratch memory, whose every access also waits for the stores issued before it)
  static_assert(TN == 2, "two column blocks");
  const int n_c0 = min(n0 + r, p.N - 1), n_c1 = min(n0 + 32 + r, p.N - 1);
  float aln0 = (XNOR && !CONV && p.alpha) ? p.alpha[n_c0] : 1.0f;
  float aln1 = (XNOR && !CONV && p.alpha) ? p.alpha[n_c1] : 1.0f;
  float thn0 = (XNOR && OUT == kOutBits && p.thr) ? p.thr[n_c0] : 0.0f;
  float thn1 = (XNOR && OUT == kOutBits && p.thr) ? p.thr[n_c1] : 0.0f;
  const int rowsum_lane = XNOR ? 0 : p.rowsum[min(m0 + lane, p.M - 1)];
  const float alpha_lane = (CONV && p.alpha) ? p.alpha[min(m0 + lane, p.M - 1)] : 1.0f;

  if (seg_lo < seg_hi) issue_segment<NA, NB, CONV>(p, stage, &voff[0][0], piece[0], piece[1], seg_lo);
  FP4_STAMP(1);
  FP4_REALTIME(4);

  v16f acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
  int pa[TM], pb[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) pa[i] = 0;
#pragma unroll
  for (int j = 0; j < TN; ++j) pb[j] = 0;

  for (int seg = seg_lo; seg < seg_hi; ++seg) {
    // the segment's words into registers (the compiler waits for the loads in flight: it tracks
    // LDS writes of the load unit)
    uint4 w[NB][2];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int g = 0; g < 2; ++g) w[b][g] = stage[b * 128 + rd[g]];
    if (8 * seg + 8 > p.Kw) {  // last segment of a row that ends inside it: words past the row are zero
#pragma unroll
      for (int g = 0; g < 2; ++g) {
        const int left = p.Kw - (8 * seg + 2 * (2 * g + h));  // valid words of this lane's piece
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          if (left < 2) w[b][g].z = w[b][g].w = 0;
          if (left < 1) w[b][g].x = w[b][g].y = 0;
        }
      }
    }
    // The next segment is requested before this one is multiplied, into the area just read.  Its
    // loads must not land on words that are still to be read, and a read that has merely been
    // issued may still wait in the LDS queue behind those of the CU's other waves when the data
    // arrives (a few hundred cycles for an L2 hit; seen as a few wrong counts in a chip-filling
    // GEMM): the reads are waited for first.  (A second area per wave used in turn, which needs
    // no wait, and two segments' loads in flight on top of that, with counted waits written out
    // because the compiler waits for every pending load of the load unit before an LDS read it
    // knows of, both measured no faster with operands that really come from HBM: 9.5 and 9.9
    // against 9.5 us on the first fully connected layer.)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#ifdef BMX_FP4_STAMPS
    if (seg == seg_lo) { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); FP4_STAMP(2); }
#endif
    if (seg + 1 < seg_hi) issue_segment<NA, NB, CONV>(p, stage, &voff[0][0], piece[0], piece[1], seg + 1);
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      const int kg = 2 * seg + g;
      if (kg < g_lo || kg >= g_hi) continue;  // wave-uniform: a range may start or end mid-segment
      if (XNOR) {
#pragma unroll
        for (int i = 0; i < TM; ++i) pa[i] = add_popcount4(pa[i], w[i][g]);
#pragma unroll
        for (int j = 0; j < TN; ++j) pb[j] = add_popcount4(pb[j], w[NA + j][g]);
      }
      uint4 hi[NB];
#pragma unroll
      for (int b = 0; b < NB; ++b)
        hi[b] = make_uint4(w[b][g].x >> 3, w[b][g].y >> 3, w[b][g].z >> 3, w[b][g].w >> 3);
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        // E8M0 block scales: planes 0 and 3 hold 0.5 (x 2), plane 1 holds 1, plane 2 holds 2 (x 1/2)
        const int sc = n == 1 ? 127 : (n == 2 ? 126 : 128);
        v8i eb[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) eb[j] = nibble_plane(w[NA + j][g], hi[NA + j], n);
        if constexpr (PL == 2) {
          // two bit planes: one operand whose nibbles hold the 2-bit value itself (E2M1 codes 0 to 3
          // = 0, 0.5, 1, 1.5; block scale 2), so a row block costs one MFMA per column block, not two
          v8i ea[TM];
#pragma unroll
          for (int i = 0; i < TM; ++i) ea[i] = nibble_pair(w[2 * i][g], w[2 * i + 1][g], n);
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
              acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ea[i], eb[j], acc[i][j], 4, 4, 0, 128, 0, sc);
        } else {
          v8i ea[NA];
#pragma unroll
          for (int b = 0; b < NA; ++b) ea[b] = nibble_plane(w[b][g], hi[b], n);
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int pl = 0; pl < PL; ++pl)
#pragma unroll
              for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ea[i * PL + pl], eb[j], acc[i][j], 4, 4, 0,
                                                                           sc + pl, 0, sc);
        }
      }
    }
  }
  FP4_STAMP(3);
  FP4_REALTIME(5);
  // The constants requested before the loop are taken in here, in one place: met for the first
  // time in the branches of the epilogue, each would get a wait of its own there, and such a
  // wait also sits out every store issued before it.
  asm volatile("" : "+v"(aln0), "+v"(aln1), "+v"(thn0), "+v"(thn1));
  int rowsum_l = rowsum_lane;
  float alpha_l = alpha_lane;
  asm volatile("" : "+v"(rowsum_l), "+v"(alpha_l));

  // CONV: where this lane's pixels' results go
  uint32_t pix_img[TN], pix_rem[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int n = min(n0 + 32 * j + r, p.N - 1);
    pix_img[j] = CONV ? fast_div((uint32_t)n, p.div_howo) : 0u;
    pix_rem[j] = CONV ? (uint32_t)n - pix_img[j] * (uint32_t)p.HoWo : 0u;
  }
  // ---- epilogue.  Register v of lane (r, h) in block (i, j) is C[32 i + 8 (v / 4) + 4 h + v % 4][32 j + r].
  // tot: the full-K sum of the MFMA results; ra, cb: pc(A row), pc(B column) over the full K
  // (plane form: ra = the row sum of the quantised activations).
  // inside: the tile lies wholly inside C (wave-uniform), so no element needs its bounds tested
  auto finish = [&](auto inside_tag, int i, int j, int v, float tot, int ra, int cb, float al, float th) {
    constexpr bool INSIDE = decltype(inside_tag)::value;
    const int mi = 32 * i + 8 * (v >> 2) + 4 * h + (v & 3);
    const int m = m0 + mi, n = n0 + 32 * j + r;
    const uint32_t idx = CONV ? (pix_img[j] * (uint32_t)p.M + (uint32_t)m) * (uint32_t)p.HoWo + pix_rem[j]
                              : (uint32_t)(m * p.ldc + n);
    if (!XNOR) {
      if (INSIDE || (m < p.M && n < p.N && live)) {
        const int sv = 2 * (int)tot - ra;
        if (p.C_i32) __builtin_nontemporal_store(sv, p.C_i32 + idx);
        if (p.C_f32) __builtin_nontemporal_store((float)sv / p.levels, p.C_f32 + idx);
      }
      return;
    }
    const float dot = (float)(p.Kreal - 2 * ra - 2 * cb) + 4.0f * tot;  // exact: integers below 2^24
    if (OUT == kOutBits) {
      // the 64-lane mask of the sign decision: its low half is 32 columns of row m, its high half
      // the same columns of the row four below
      const uint64_t mask = __ballot(live && n < p.N && al * dot >= th);
      if (r == 0 && m < p.M && live)
        p.C_bits[(uint32_t)(m * (2 * p.ldc) + (n >> 5))] = h ? (uint32_t)(mask >> 32) : (uint32_t)mask;
    } else if (INSIDE || (m < p.M && n < p.N && live)) {
      if (OUT == kOutI32) __builtin_nontemporal_store(p.as_count ? ((int)dot + p.Kreal) >> 1 : (int)dot, p.C_i32 + idx);
      else __builtin_nontemporal_store(al * dot, p.C_f32 + idx);
    }
  };
  // popcounts: a lane counted its half of K for row / column r; the other half sits 32 lanes away
  if (XNOR) {
#pragma unroll
    for (int i = 0; i < TM; ++i) pa[i] += __shfl_xor(pa[i], 32);
#pragma unroll
    for (int j = 0; j < TN; ++j) pb[j] += __shfl_xor(pb[j], 32);
  }

  if (!SPLIT) {
    // the row terms of every result register first (a shuffle each: fetched one by one between
    // the stores, each would cost an LDS round trip), then nothing but arithmetic and stores
    int ra[TM][16];
    float alm[TM][16];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int mi = 32 * i + 8 * (v >> 2) + 4 * h + (v & 3);
        ra[i][v] = XNOR ? __shfl(pa[i], mi & 31) : __shfl(rowsum_l, mi);
        alm[i][v] = CONV ? __shfl(alpha_l, mi) : 1.0f;
      }
    auto store_tile = [&](auto inside_tag) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            finish(inside_tag, i, j, v, acc[i][j][v], ra[i][v], pb[j], CONV ? alm[i][v] : (j ? aln1 : aln0), j ? thn1 : thn0);
    };
    if (m0 + 32 * TM <= p.M && n0 + 32 * TN <= p.N) store_tile(std::true_type{});
    else store_tile(std::false_type{});
    return;
  }

  // ---- K split: every wave writes its partial tile and its popcounts over its own staging
  // areas (nothing of another wave's lies there), then finishes the accumulator groups
  // g = wave, wave + S, ... : S partials in, one store out.
  float4* part = (float4*)lds;
  uint2* part16 = (uint2*)lds;  // HALF: four sums as two fp16 pairs, 8 bytes per lane and group
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int g = (i * TN + j) * 4 + q;
        if constexpr (HALF) {
          const half2_t lo = __builtin_amdgcn_cvt_pkrtz(acc[i][j][4 * q], acc[i][j][4 * q + 1]);
          const half2_t hi = __builtin_amdgcn_cvt_pkrtz(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
          part16[(wave * kSlot) * 2 + g * 64 + lane] = make_uint2(__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi));
        } else {
          part[wave * kSlot + g * 64 + lane] =
              make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        }
      }
  int* cnt = (int*)(part + wave * kSlot + kPart);  // [32 TM] row counts, [32 TN] column counts
  if (XNOR && h == 0) {
#pragma unroll
    for (int i = 0; i < TM; ++i) cnt[32 * i + r] = pa[i];
#pragma unroll
    for (int j = 0; j < TN; ++j) cnt[32 * TM + 32 * j + r] = pb[j];
  }
  __syncthreads();
  FP4_STAMP(4);
  // FULL: all eight waves split K (the usual case): no partial has to be masked out
  auto reduce = [&](auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    // full-K popcounts: lane l sums row l of the tile (TM = 2: 64 rows) and column l over the S
    // waves' counts, one conflict-free read each; a lane then picks the rows and the column of
    // its own results out of other lanes' registers
    int pa_tot = rowsum_l, pb_tot = 0;  // (plane form: the row sum stands where the row count would)
    if (XNOR) {
      static_assert((TM == 2 && TN == 2) || !SPLIT, "one lane per row and per column of the tile");
      int ca[8], cb8[8];
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const int* c = (const int*)(part + (FULL || s < S ? s : S - 1) * kSlot + kPart);
        ca[s] = c[lane];
        cb8[s] = c[32 * TM + lane];
      }
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        pa_tot += (FULL || s < S) ? ca[s] : 0;
        pb_tot += (FULL || s < S) ? cb8[s] : 0;
      }
    }
    // the popcount terms, scale and stores of accumulator group g, whose four sums are tot
    auto finish_group = [&](int g, float4 tot) {
      const int blk = g >> 2, q = g & 3, i = blk / TN, j = blk % TN;
      const int row0 = 32 * i + 8 * q + 4 * h;  // this lane's four rows: row0 .. row0 + 3
      int ra[4], cb = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) ra[e] = __shfl(pa_tot, row0 + e);
      if (XNOR) cb = __shfl(pb_tot, 32 * j + r);
      const float al = j == 0 ? aln0 : aln1, th = j == 0 ? thn0 : thn1;
      float alm[4] = {al, al, al, al};
      if (CONV) {
#pragma unroll
        for (int e = 0; e < 4; ++e) alm[e] = __shfl(alpha_l, row0 + e);
      }
      finish(std::false_type{}, i, j, 4 * q, tot.x, ra[0], cb, alm[0], th);
      finish(std::false_type{}, i, j, 4 * q + 1, tot.y, ra[1], cb, alm[1], th);
      finish(std::false_type{}, i, j, 4 * q + 2, tot.z, ra[2], cb, alm[2], th);
      finish(std::false_type{}, i, j, 4 * q + 3, tot.w, ra[3], cb, alm[3], th);
    };
    if constexpr (FULL && HALF) {
      // Eight waves, fp16 partials (the fully connected layers): a wave has exactly kGroups / 8
      // groups, and the partials of all of them are requested before the first is summed, so
      // that the second group's LDS round trip runs under the first group's sums and stores.
      constexpr int NG = kGroups / 8;
      uint2 t[NG][8];
#pragma unroll
      for (int it = 0; it < NG; ++it)
#pragma unroll
        for (int s = 0; s < 8; ++s) t[it][s] = part16[(s * kSlot) * 2 + (wave + 8 * it) * 64 + lane];
#pragma unroll
      for (int it = 0; it < NG; ++it) {
        float4 tot = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          // v_dot2_f32_f16 with (1, 0) or (0, 1) picks a half, widens it and adds it in one
          // instruction (exact: whole numbers up to 2048, fp32 accumulation)
          const half2_t lo = __builtin_bit_cast(half2_t, t[it][s].x), hi = __builtin_bit_cast(half2_t, t[it][s].y);
          const half2_t first = {(__fp16)1.0f, (__fp16)0.0f}, second = {(__fp16)0.0f, (__fp16)1.0f};
          tot.x = __builtin_amdgcn_fdot2(lo, first, tot.x, false);
          tot.y = __builtin_amdgcn_fdot2(lo, second, tot.y, false);
          tot.z = __builtin_amdgcn_fdot2(hi, first, tot.z, false);
          tot.w = __builtin_amdgcn_fdot2(hi, second, tot.w, false);
        }
#ifdef BMX_FP4_STAMPS
        if (it == 0) { FP4_STAMP(7); }
#endif
        finish_group(wave + 8 * it, tot);
      }
      return;
    }
    for (int g = wave; g < kGroups; g += S) {
      // all reads first (partials past S repeat the last one and count as nothing), so that the
      // LDS round trips overlap instead of adding up
      float4 tot = make_float4(0.f, 0.f, 0.f, 0.f);
      if constexpr (HALF) {
        uint2 t[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) t[s] = part16[((FULL || s < S ? s : S - 1) * kSlot) * 2 + g * 64 + lane];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          const bool on = FULL || s < S;
          const half2_t lo = __builtin_bit_cast(half2_t, t[s].x), hi = __builtin_bit_cast(half2_t, t[s].y);
          tot.x += on ? (float)lo[0] : 0.f;
          tot.y += on ? (float)lo[1] : 0.f;
          tot.z += on ? (float)hi[0] : 0.f;
          tot.w += on ? (float)hi[1] : 0.f;
        }
      } else {
        float4 t[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) t[s] = part[(FULL || s < S ? s : S - 1) * kSlot + g * 64 + lane];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          const bool on = FULL || s < S;
          tot.x += on ? t[s].x : 0.f;
          tot.y += on ? t[s].y : 0.f;
          tot.z += on ? t[s].z : 0.f;
          tot.w += on ? t[s].w : 0.f;
        }
      }
#ifdef BMX_FP4_STAMPS
      if (g == wave) { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); FP4_STAMP(7); }
#endif
      finish_group(g, tot);
    }
  };
  if (S == 8) reduce(std::true_type{});
  else reduce(std::false_type{});
  FP4_STAMP(5);
#ifdef BMX_FP4_STAMPS
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  FP4_STAMP(6);
#endif
}

}  // namespace
int gemm_fp4_half = 0;  // 2 = keep fp32 partials (tests of both forms)
namespace {

template <int TM, int TN, int PL, bool XNOR, int OUT, bool SPLIT, bool HALF, bool CONV>
hipError_t launch_tile(const Fp4Params& p, int S, int tiles_per_wg, int64_t blocks, hipStream_t s) {
  constexpr int NB = TM * PL + TN, kStage = NB * 128, kGroups = TM * TN * 4, kCnt = (TM + TN) * 8;
  constexpr int part = HALF ? kGroups * 32 : kGroups * 64;
  constexpr int slot = (!SPLIT || kStage > part + kCnt) ? kStage : part + kCnt;
  const int waves = SPLIT ? S : tiles_per_wg;
  const size_t lds = (size_t)waves * slot * 16;
  auto kern = gemm_fp4_kernel<TM, TN, PL, XNOR, OUT, SPLIT, HALF, CONV>;
  if (lds > 64 * 1024) {  // more than the default limit of dynamic LDS: raised once per device
    static bool raised[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!raised[dev]) {
      const hipError_t e =
          hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e != hipSuccess) return e;
      raised[dev] = true;
    }
  }
  note_kernel("gemm_fp4_kernel<%d,%d,%d,%s,%s%s> grid %lld x %d, K split %d%s, fp4", TM, TN, PL, XNOR ? "xnor" : "planes",
              !XNOR ? "S" : (OUT == kOutF32 ? "f32" : (OUT == kOutI32 ? "i32" : "bits")), CONV ? ",conv" : "",
              (long long)blocks, 64 * waves, SPLIT ? S : 1, HALF ? " (fp16 partials)" : "");
#ifdef BMX_FP4_STAMPS
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * waves), lds, s, p, S, fp4_stamps);
#else
  hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(64 * waves), lds, s, p, S);
#endif
  return hipGetLastError();
}

}  // namespace
int gemm_fp4_band = 0;  // 0 = automatic (16), else rows of tiles per band of the tile order
namespace {

void set_tile_order(Fp4Params& p) {
  p.band = gemm_fp4_band > 0 ? std::min(gemm_fp4_band, p.tiles_m) : std::min(16, p.tiles_m);
  p.per_band = p.band * p.tiles_n;
  p.last_band = (p.tiles_m - 1) / p.band;
  p.last_rows = p.tiles_m - p.last_band * p.band;
  p.div_per_band = make_fast_div((uint32_t)p.per_band);
  p.div_band = make_fast_div((uint32_t)p.band);
  p.div_last = make_fast_div((uint32_t)p.last_rows);
}

template <int PL, bool XNOR, int OUT, bool CONV = false>
hipError_t launch_split(const Fp4Params& p, int S, int tiles_per_wg, int64_t blocks, hipStream_t s) {
  if (S > 1) {
    // a wave's partial sums are at most (its bits of K) x (2^PL - 1): whole numbers up to 2048
    // are exact in fp16
    const int64_t most = (int64_t)(p.g_base + (p.g_rem ? 1 : 0)) * 256 * ((1 << PL) - 1);
    if (most <= 2048 && gemm_fp4_half != 2)
      return launch_tile<2, 2, PL, XNOR, OUT, true, true, CONV>(p, S, tiles_per_wg, blocks, s);
    return launch_tile<2, 2, PL, XNOR, OUT, true, false, CONV>(p, S, tiles_per_wg, blocks, s);
  }
  return launch_tile<2, 2, PL, XNOR, OUT, false, false, CONV>(p, S, tiles_per_wg, blocks, s);
}

}  // namespace

int gemm_fp4_split = 0;  // 0 = automatic; settable for sweeps and for the tests of every split
int gemm_fp4_tall = 0;   // 0 = automatic; 1 = never 128 x 64 of C per wave; 2 = wherever the form exists

// Takes the problem when both operands have 16-byte aligned rows, sums stay exact in fp32, the
// operands can be addressed with 32-bit byte offsets, and there are enough 64 x 64 tiles for
// the tile shape to pay; false otherwise (the caller then uses the 32 x 32 kernel).
bool launch_gemm_fp4(const uint64_t* A, int64_t lda_w, int planes, const int32_t* rowsum, const uint64_t* B,
                     int64_t ldb_w, int M, int N, int K, const float* alpha_n, int32_t* C_i32, float* C_f32,
                     uint64_t* C_bits, const float* thr_n, int64_t ldc, bool as_count, hipStream_t s,
                     hipError_t* err) {
  if (gemm_engine == 1 || gemm_engine == 2 || gemm_engine == 4) return false;
  if (planes < 1 || planes > 2) return false;
  if ((lda_w & 1) || (ldb_w & 1) || ((uintptr_t)A & 15) || ((uintptr_t)B & 15)) return false;
  if ((int64_t)K * ((1 << planes) - 1) >= ((int64_t)1 << 24)) return false;
  if ((int64_t)M * planes * lda_w * 8 >= ((int64_t)1 << 32) || (int64_t)N * ldb_w * 8 >= ((int64_t)1 << 32))
    return false;
  // (outputs are addressed with 32-bit element indices, rows rounded up to whole tiles)
  if (((int64_t)M + 64) * ldc * (C_bits ? 2 : 1) >= ((int64_t)1 << 31)) return false;
  const int tiles_m = (int)ceil_div(M, 64), tiles_n = (int)ceil_div(N, 64);
  const int64_t tiles = (int64_t)tiles_m * tiles_n;
  if (gemm_engine != 5 && tiles < 64) return false;
  if (tiles >= ((int64_t)1 << 28)) return false;
  Fp4Params p;
  p.A = A;
  p.B = B;
  p.lda_bytes = (uint32_t)(lda_w * 8);
  p.ldb_bytes = (uint32_t)(ldb_w * 8);
  p.M = M;
  p.N = N;
  p.Kw = (int)words_for(K);
  p.Kreal = K;
  const int ngroups = (int)ceil_div(p.Kw, 4);
  p.tiles_m = tiles_m;
  p.tiles_n = tiles_n;
  set_tile_order(p);
  p.alpha = alpha_n;
  p.thr = thr_n;
  p.rowsum = rowsum;
  p.levels = (float)((1u << planes) - 1u);
  p.as_count = as_count ? 1 : 0;
  p.C_i32 = C_i32;
  p.C_f32 = C_f32;
  p.C_bits = (uint32_t*)C_bits;
  p.ldc = (int)ldc;
  p.HoWo = p.Wo = p.Hp = p.Wpp = p.Cw = p.stride = 1;
  p.run_pieces = p.row_bytes = p.npieces = 1;
  p.div_howo = p.div_wo = p.div_run = make_fast_div(1);
  // K split: about two waves per SIMD (2048 in all), at most eight per tile, and every wave
  // keeps at least one 64-byte segment
  int S = gemm_fp4_split;
  if (S <= 0) {
    S = (int)(2048 / tiles);
    S = S > 8 ? 8 : S;
  }
  S = S > 8 ? 8 : S;
  if (S > ngroups / 2) S = ngroups / 2;
  if (S < 1) S = 1;
  p.g_base = ngroups / S;
  p.g_rem = ngroups - p.g_base * S;
  const int tiles_per_wg = 4;
  // Chip-filling xnor products without a split: 128 x 64 of C per wave.  Six expanded operand
  // blocks then serve eight MFMAs instead of four serving four: 4.5 VALU instructions per MFMA
  // instead of 6, in a loop that the vector ALU's issue slot bounds, not the matrix pipe.  The
  // form needs 231 registers, so two waves share a SIMD where three of the square form do, and
  // the two come out level except where a SIMD works through many tiles (half as many tile
  // starts and ends per MFMA): 8192^3 214 against 222 us, 4096^3 38.6 against 34.1 us.  Taken
  // from four rounds of tiles on.
  if (planes == 1 && rowsum == nullptr && !C_bits && S == 1 && gemm_fp4_tall != 1 &&
      (gemm_fp4_tall == 2 || ceil_div(M, 128) * (int64_t)tiles_n >= 8192) &&
      ((int64_t)M + 128) * ldc < ((int64_t)1 << 31)) {
    p.tiles_m = (int)ceil_div(M, 128);
    set_tile_order(p);
    p.tiles_per_xcd = (int)ceil_div(ceil_div((int64_t)p.tiles_m * tiles_n, tiles_per_wg), 8);
    const int64_t tall_blocks = 8 * (int64_t)p.tiles_per_xcd;
    if (C_i32) *err = launch_tile<4, 2, 1, true, kOutI32, false, false, false>(p, 1, tiles_per_wg, tall_blocks, s);
    else *err = launch_tile<4, 2, 1, true, kOutF32, false, false, false>(p, 1, tiles_per_wg, tall_blocks, s);
    return true;
  }
  const int64_t wgs = S > 1 ? tiles : ceil_div(tiles, tiles_per_wg);
  p.tiles_per_xcd = (int)ceil_div(wgs, 8);
  const int64_t blocks = 8 * (int64_t)p.tiles_per_xcd;
  if (planes == 1 && rowsum == nullptr) {
    if (C_bits) *err = launch_split<1, true, kOutBits>(p, S, tiles_per_wg, blocks, s);
    else if (C_i32) *err = launch_split<1, true, kOutI32>(p, S, tiles_per_wg, blocks, s);
    else *err = launch_split<1, true, kOutF32>(p, S, tiles_per_wg, blocks, s);
  } else if (planes == 1) {
    *err = launch_split<1, false, kOutF32>(p, S, tiles_per_wg, blocks, s);
  } else {
    *err = launch_split<2, false, kOutF32>(p, S, tiles_per_wg, blocks, s);
  }
  return true;
}

// The convolution on the same kernel (Xp, Wp as for launch_binary_conv2d).  Takes the problem when
// every 16-byte piece of an im2col row is 16 consecutive bytes of the packed image (an even number
// of channel words), rows are 16-byte aligned, and image and output fit 32-bit offsets.
bool launch_conv_fp4(const uint64_t* Xp, int Nimg, int C, int H, int W, const uint64_t* Wp, int O, int KH, int KW,
                     int stride, int pad, const float* alpha, int32_t* out_i32, float* out_f32, hipStream_t s,
                     hipError_t* err) {
  if (gemm_engine == 1 || gemm_engine == 2 || gemm_engine == 4) return false;
  const int Ho = (H + 2 * pad - KH) / stride + 1;
  const int Wo = (W + 2 * pad - KW) / stride + 1;
  const int Cw = (int)words_for(C);
  const int kwords = KH * KW * Cw;
  const int64_t ld_words = conv_weight_row_words(kwords);
  const int64_t P = (int64_t)Nimg * Ho * Wo;
  const int Hp = H + 2 * pad, Wpp = W + 2 * pad;
  if ((Cw & 1) || (ld_words & 1) || ((uintptr_t)Wp & 15) || ((uintptr_t)Xp & 15)) return false;
  if ((int64_t)kwords * 64 >= ((int64_t)1 << 24)) return false;
  if ((int64_t)Nimg * Hp * Wpp * Cw * 8 >= ((int64_t)1 << 32) || (int64_t)O * ld_words * 8 >= ((int64_t)1 << 32))
    return false;
  if (P >= ((int64_t)1 << 31) || ((int64_t)Nimg * O + 64) * Ho * Wo >= ((int64_t)1 << 31)) return false;
  const int tiles_m = (int)ceil_div(O, 64), tiles_n = (int)ceil_div(P, 64);
  const int64_t tiles = (int64_t)tiles_m * tiles_n;
  if (tiles >= ((int64_t)1 << 28)) return false;
  Fp4Params p;
  p.A = Wp;
  p.B = Xp;
  p.lda_bytes = (uint32_t)(ld_words * 8);
  p.ldb_bytes = 0;
  p.M = O;
  p.N = (int)P;
  p.Kw = kwords;
  p.Kreal = C * KH * KW;
  const int ngroups = (int)ceil_div(kwords, 4);
  p.tiles_m = tiles_m;
  p.tiles_n = tiles_n;
  set_tile_order(p);
  p.alpha = alpha;
  p.thr = nullptr;
  p.rowsum = nullptr;
  p.levels = 1.0f;
  p.as_count = 0;
  p.C_i32 = out_i32;
  p.C_f32 = out_f32;
  p.C_bits = nullptr;
  p.ldc = 0;
  p.HoWo = Ho * Wo;
  p.Wo = Wo;
  p.Hp = Hp;
  p.Wpp = Wpp;
  p.Cw = Cw;
  p.stride = stride;
  p.run_pieces = (uint32_t)(KW * Cw / 2);
  p.row_bytes = (uint32_t)((int64_t)Wpp * Cw * 8);
  p.npieces = (uint32_t)(kwords / 2);
  p.div_howo = make_fast_div((uint32_t)(Ho * Wo));
  p.div_wo = make_fast_div((uint32_t)Wo);
  p.div_run = make_fast_div(p.run_pieces);
  // K split: about two waves per SIMD; a wave may carry a single group of 256 bits
  int S = gemm_fp4_split;
  if (S <= 0) S = (int)ceil_div(2048, tiles);
  S = S > 8 ? 8 : S;
  if (S > ngroups) S = ngroups;
  if (S < 1) S = 1;
  p.g_base = ngroups / S;
  p.g_rem = ngroups - p.g_base * S;
  const int tiles_per_wg = 4;
  const int64_t wgs = S > 1 ? tiles : ceil_div(tiles, tiles_per_wg);
  p.tiles_per_xcd = (int)ceil_div(wgs, 8);
  const int64_t blocks = 8 * (int64_t)p.tiles_per_xcd;
  if (out_i32) *err = launch_split<1, true, kOutI32, true>(p, S, tiles_per_wg, blocks, s);
  else *err = launch_split<1, true, kOutF32, true>(p, S, tiles_per_wg, blocks, s);
  return true;
}

}  // namespace bmx
