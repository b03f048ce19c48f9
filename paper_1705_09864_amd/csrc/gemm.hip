// xor/and + popcount GEMM on packed operands (VALU integer bound), and the implicit-GEMM
// convolution that runs on the same kernel.
// Paper: Sec. 2.2.1 (xnor GEMM on packed words), Sec. 2.2.2 / Eq. 2 (output form), Sec. 2.1
// Eq. 1 for the bit-plane variant, Sec. 3.1 for the convolution as a GEMM (M = filters,
// N = batch * output pixels, K = kh * kw * C).
//
// C[m][n] = f(sum_k popcount(A[m][k] op B[n][k])), both operands packed along K.
//
// Shape of the kernel.  Lanes span 64 consecutive columns n, so C rows are written
// coalesced.  A lane keeps a chunk of CH (32 or 24) dwords of its own B row in registers
// ("B stationary") and the wave streams rows of A past it: an A row chunk is the same for
// every lane, so it is fetched with two scalar loads into SGPRs and enters v_xor_b32 /
// v_and_b32 as the scalar source.  One row step is 2 * CH VALU instructions (v_xor +
// v_bcnt, the popcount instruction also accumulates) against 4 * CH bytes of scalar loads
// and nothing else; the scalar loads of the next row are in flight while the current one is
// consumed.  A wave owns R rows (one accumulator register per row) and a contiguous range of
// K chunks; the S waves of a workgroup split K between them and add their partial counts
// through LDS at the end.  Splitting K is what gives a skinny problem (a few hundred rows)
// enough waves to keep four per SIMD, which the VALU needs to issue at full rate.
//
// GEMM mode: the B chunk of a wave (64 rows x 128 bytes) is read with coalesced 16-byte
// loads and transposed through a wave-private LDS tile (with 32 rows per wave it is also
// prefetched one chunk ahead; the leaner shapes rely on the other waves of the SIMD).
//
// Convolution mode: column n is output pixel n (flat over image, row, column), its B row is
// the im2col row of that pixel, which is never formed: word j of it is word (j mod Cw) of tap
// (j div Cw) and is gathered straight from the halo-padded channel-packed image, 8 bytes per
// lane and word (neighbouring lanes are neighbouring pixels, so the gather is coalesced; the
// offset of a word is the same for every lane and is tracked on the scalar unit).
// A is the filter matrix, rows zero padded to whole chunks.
//
// Bit planes (k-bit activations): plane p of row m is virtual row m * planes + p of A, so
// the main loop is unaware of planes; the final reduction weights plane p by 2^p.
#include <type_traits>

#include "bmx_internal.h"
#include "scalar_stream.h"

namespace bmx {

int gemm_tune_rows = 0;    // 0 = automatic; otherwise force R (8, 16 or 32)
int gemm_tune_ksplit = 0;  // 0 = automatic; otherwise force the number of K-split waves
int gemm_tune_order = 0;   // 1 = row blocks fastest over the workgroup id

namespace {

constexpr int kChunk = 32;  // dwords of K per register chunk in GEMM mode
constexpr int kTRow = 36;   // LDS row stride of the transposition tile (dwords, 16-byte multiple)
constexpr int kTileDw = 64 * kTRow;

enum GemmOut { kGemmI32 = 0, kGemmF32 = 1, kGemmF32Alpha = 2, kGemmPlanes = 3, kGemmBits = 4 };

struct GemmParams {
  const uint32_t* A;      // [Mv][lda] dwords, virtual rows (row m, plane p -> m * planes + p)
  const uint32_t* B;      // GEMM: [N][ldb] dwords.  Convolution: the packed image Xp
  int64_t lda, ldb;       // dwords
  int Mv, N;
  int planes;             // 1 in xor mode
  int rows_per_block;     // virtual rows per workgroup, a multiple of planes, <= R
  int nch;                // chunks the main loop covers; A rows are readable up to nch * CH dwords
  int Kd;                 // dwords of a B row that may be read (the rest of a chunk reads as 0)
  int tail0, tail1;       // dword range finished in the epilogue with plain loads (may be empty)
  int Kreal;              // K in bits (xor modes)
  const int32_t* rowsum;  // planes mode: sum_k q[m][k]
  const float* alpha;     // GEMM: per column n.  Convolution: per row (filter) m
  int as_count;           // kGemmI32: store the xnor count (dot + K) / 2 instead of the dot product
  const float* thr;       // kGemmBits: per column n threshold of the sign decision, or null (0)
  float levels;           // planes mode: 2^bits - 1
  int32_t* C_i32;
  float* C_f32;
  uint64_t* C_bits;       // kGemmBits: packed sign of the scaled result, ldc words per row
  int64_t ldc;            // GEMM: elements between C rows.  Convolution: Ho * Wo
  int out;                // GemmOut
  int row_blocks;         // ceil(Mv / rows_per_block)
  int rows_fastest;       // tuning: row blocks fastest over the workgroup id instead
  // convolution geometry (N = images * Ho * Wo output pixels, Mv = O filters)
  int HoWo, Wo, Hp, Wp_pix, Cw, stride, KWid;
  FastDiv div_howo, div_wo, div_rw;  // div_rw: by KW * Cw, the words of one kernel row
};

// One CH-dword chunk of an A row in SGPRs: ordinary loads through the constant address space
// from a wave-uniform address, so the compiler emits the scalar loads, waits for them and keeps
// their registers itself (see ScalarSeg for how the pipeline order is expressed).
template <int CH>
struct ARow {
  static_assert(CH == 32 || CH == 24, "chunk is two scalar loads: 16 + 16 or 16 + 8 dwords");
  u32x16 lo;
  typename std::conditional<CH == 32, u32x16, u32x8>::type hi;
  __device__ __forceinline__ void issue(const_u32_ptr src) {
    lo = *(const_u32x16_ptr)src;
    if constexpr (CH == 32) hi = *(const_u32x16_ptr)(src + 16);
    else hi = *(const_u32x8_ptr)(src + 16);
  }
  // The chunk's first use (the compiler's wait goes in front of it); `next`, the address of the
  // request that follows, is defined here, so that request stays below this point.
  __device__ __forceinline__ void landed(const_u32_ptr& next) {
    asm volatile("" : "+s"(lo), "+s"(next));
    asm volatile("" : "+s"(hi), "+s"(next));
  }
  template <int J>
  __device__ __forceinline__ uint32_t get() const {
    if constexpr (J < 16) return lo[J];
    else return hi[J - 16];
  }
};

template <int CH, bool OP_AND, int J = 0>
__device__ __forceinline__ void row_popcount(const ARow<CH>& a, const uint32_t (&b)[CH], int& acc) {
  if constexpr (J < CH) {
    const uint32_t av = a.template get<J>();
    acc += __builtin_popcount(OP_AND ? (b[J] & av) : (b[J] ^ av));
    asm volatile("" : "+v"(acc));  // keep the op / popcount-accumulate pairs as written
    row_popcount<CH, OP_AND, J + 1>(a, b, acc);
  }
}

// The R row steps of one chunk, unrolled so that every accumulator has a fixed register.
// Invariant on entry of step r: the loads of row r are in flight in buf[r & 1].
template <int R, int CH, bool OP_AND, int r = 0>
__device__ __forceinline__ void row_steps(ARow<CH> (&buf)[2], const uint32_t (&b)[CH], int (&acc)[R],
                                          const_u32_ptr& src, uint64_t row_bytes, int& rows_valid,
                                          const_u32_ptr next_chunk_row0) {
  if constexpr (r < R) {
    // The next request: the next row of this chunk (rows past the block's last valid row repeat
    // it), or row 0 of the wave's next chunk after the last row.
    // (the select is kept opaque so that it stays two scalar instructions per row instead
    // of R loop-invariant values that would not fit the scalar register file)
    if constexpr (r + 1 < R) {
      asm volatile("" : "+s"(rows_valid));
      src = (const_u32_ptr)((uint64_t)src + ((r + 1 < rows_valid) ? row_bytes : (uint64_t)0));
    } else {
      src = next_chunk_row0;
    }
    buf[r & 1].landed(src);
    buf[(r + 1) & 1].issue(src);
    row_popcount<CH, OP_AND>(buf[r & 1], b, acc[r]);
    row_steps<R, CH, OP_AND, r + 1>(buf, b, acc, src, row_bytes, rows_valid, next_chunk_row0);
  }
}

template <int R, int CH, bool OP_AND, bool PF, bool CONV>
__global__ void __launch_bounds__(512, PF ? 4 : 6)
gemm_kernel(const GemmParams p) {
  static_assert(R % 2 == 0, "buffer parity must repeat from chunk to chunk");
  static_assert(CONV || CH == kChunk, "the LDS transposition tile is laid out for 32-dword chunks");
  static_assert(!(CONV && PF), "the gather has no staging registers to prefetch into");
  extern __shared__ __align__(16) uint32_t lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int S = __builtin_amdgcn_readfirstlane((int)(blockDim.x >> 6));
  // Column blocks vary fastest over the linear workgroup id (measured faster than the
  // other order on the FC shapes: neighbouring workgroups stream the same A rows).
  const int col_blocks = (p.N + 63) / 64;
  const int rb = p.rows_fastest ? (int)(blockIdx.x % p.row_blocks) : (int)(blockIdx.x / col_blocks);
  const int cb = p.rows_fastest ? (int)(blockIdx.x / p.row_blocks) : (int)(blockIdx.x % col_blocks);
  const int n0 = cb * 64;
  const int m0 = rb * p.rows_per_block;  // first virtual row of the block
  int rows_valid = min(p.rows_per_block, p.Mv - m0);
  const int c0 = (int)((int64_t)wave * p.nch / S);
  const int c1 = (int)((int64_t)(wave + 1) * p.nch / S);
  const int n = n0 + lane;
  const int nc = min(n, p.N - 1);

  // Convolution: where pixel nc sits in the packed image and in the NCHW output.
  uint32_t xoff = 0;      // byte offset of the pixel's receptive field in Xp
  int64_t lane_off = nc;  // element offset of (row 0, column n) in C; rows are ldc apart
  if constexpr (CONV) {
    const uint32_t img = fast_div((uint32_t)nc, p.div_howo);
    const uint32_t rem = (uint32_t)nc - img * (uint32_t)p.HoWo;
    const uint32_t ho = fast_div(rem, p.div_wo);
    const uint32_t wo = rem - ho * (uint32_t)p.Wo;
    xoff = (((img * (uint32_t)p.Hp + ho * (uint32_t)p.stride) * (uint32_t)p.Wp_pix +
             wo * (uint32_t)p.stride) * (uint32_t)p.Cw) * 8u;
    lane_off = (int64_t)img * p.Mv * p.HoWo + rem;
  }

  int acc[R];
#pragma unroll
  for (int r = 0; r < R; ++r) acc[r] = 0;

  if (c0 < c1) {
    // ---- GEMM B chunk loader: lane -> (row within 8, 16-byte piece of the 128-byte chunk)
    const int srow = lane >> 3, spiece = lane & 7;
    const uint32_t* bsrc[8];
    uint4 stage[8];
    if constexpr (!CONV) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
        bsrc[i] = p.B + (int64_t)min(n0 + i * 8 + srow, p.N - 1) * p.ldb + spiece * 4;
    }
    auto fetch = [&](int c) {
      if ((c + 1) * kChunk <= p.Kd) {  // whole chunk inside the rows (wave-uniform)
#pragma unroll
        for (int i = 0; i < 8; ++i) stage[i] = *(const uint4*)(bsrc[i] + c * kChunk);
      } else {  // last chunk: dwords past the row read as zero (Kd is even)
        const int left = p.Kd - (c * kChunk + spiece * 4);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          uint4 v = make_uint4(0, 0, 0, 0);
          if (left >= 4) {
            v = *(const uint4*)(bsrc[i] + c * kChunk);
          } else if (left >= 2) {
            const uint2 h = *(const uint2*)(bsrc[i] + c * kChunk);
            v.x = h.x;
            v.y = h.y;
          }
          stage[i] = v;
        }
      }
    };
    uint32_t* tile = lds + wave * kTileDw;
    // ---- convolution B chunk loader.  Word j of the im2col row is word j % rw of kernel row
    // j / rw (rw = KW * Cw words, contiguous both in K order and in the packed image), so the
    // chunk is walked with a running (word in row, byte offset) pair: one division per chunk.
    const char* xbase = (const char*)p.B;
    const uint32_t rw = (uint32_t)(p.KWid * p.Cw);
    const uint32_t row_skip = (uint32_t)(p.Wp_pix * p.Cw) * 8u - rw * 8u;  // end of row -> next row
    auto gather = [&](int c, uint32_t (&b)[CH]) {
      const uint32_t j0 = (uint32_t)c * (CH / 2);  // wave-uniform
      const uint32_t kh = fast_div(j0, p.div_rw);
      uint32_t r = j0 - kh * rw;
      uint32_t off = kh * (uint32_t)(p.Wp_pix * p.Cw) * 8u + r * 8u;
      const bool whole = (int)(2 * j0 + CH) <= p.Kd;  // no word of the chunk is padding
#pragma unroll
      for (int i = 0; i < CH / 2; ++i) {
        uint64_t v = 0;
        if (whole || (int)(2 * (j0 + i)) < p.Kd) v = *(const uint64_t*)(xbase + off + xoff);
        b[2 * i] = (uint32_t)v;
        b[2 * i + 1] = (uint32_t)(v >> 32);
        r += 1;
        off += 8;
        if (r == rw) {
          r = 0;
          off += row_skip;
        }
      }
    };

    // ---- A stream (wave-uniform addresses)
    const uint64_t row_bytes = (uint64_t)p.lda * 4;
    const uint64_t arow0 = uniform_addr((uint64_t)(uintptr_t)p.A + (int64_t)m0 * p.lda * 4);
    ARow<CH> buf[2];
    const_u32_ptr src = (const_u32_ptr)(arow0 + (uint64_t)c0 * (CH * 4));
    buf[0].issue(src);
    // Lane r touches row r of the chunk that comes next, so that the scalar loads of a row
    // step find their line in L2 instead of paying a cold miss each (the first pass over
    // a block would otherwise cost one memory round trip per row).
    const uint32_t* warm_row = p.A + (int64_t)(m0 + min(lane, rows_valid - 1)) * p.lda;
    uint32_t warm = warm_row[(int64_t)c0 * CH];
    if (PF) fetch(c0);
    for (int c = c0; c < c1; ++c) {
      uint32_t b[CH];
      if constexpr (CONV) {
        gather(c, b);
      } else {
        if (!PF) fetch(c);
        // transpose the staged chunk: row n of the tile is lane n's 32 dwords
#pragma unroll
        for (int i = 0; i < 8; ++i) *(uint4*)(tile + (i * 8 + srow) * kTRow + spiece * 4) = stage[i];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const uint4 v = *(const uint4*)(tile + lane * kTRow + j * 4);
          b[4 * j] = v.x;
          b[4 * j + 1] = v.y;
          b[4 * j + 2] = v.z;
          b[4 * j + 3] = v.w;
        }
        if (PF && c + 1 < c1) fetch(c + 1);
      }
      const int cn = min(c + 1, c1 - 1);  // after the last chunk the last row 0 is fetched again
      const const_u32_ptr next_row0 = (const_u32_ptr)(arow0 + (uint64_t)cn * (CH * 4));
      asm volatile("" ::"v"(warm));  // consume the previous touch
      warm = warm_row[(int64_t)cn * CH];
      row_steps<R, CH, OP_AND>(buf, b, acc, src, row_bytes, rows_valid, next_row0);
    }
    // The last request (row 0 of the last chunk again) is never used.
    asm volatile("" ::"v"(warm));
  }

  // Per-column scale (GEMM) in every lane; per-row values (the filter's alpha of a
  // convolution, the row sum of the plane mode) are fetched once, row i of the block into
  // lane i, and handed out with readlane: a load per row would put one memory round trip
  // after the other.
  float al = 1.0f;
  if (!CONV && (p.out == kGemmF32Alpha || p.out == kGemmBits) && p.alpha) al = p.alpha[nc];
  float th = 0.0f;
  if (!CONV && p.out == kGemmBits && p.thr) th = p.thr[nc];
  const int rows_out = rows_valid / p.planes;
  const int64_t mbase = m0 / p.planes;
  float row_alpha = 1.0f;
  int row_sum = 0;
  if (CONV && p.out == kGemmF32Alpha && lane < rows_out) row_alpha = p.alpha[mbase + lane];
  if (p.out == kGemmPlanes && lane < rows_out) row_sum = p.rowsum[mbase + lane];
  auto finish = [&](int lr, int total) {  // count of the block's output row lr -> C[m][n]
    const int64_t m = mbase + lr;
    if (p.out == kGemmBits) {
      // the 64-lane mask of (scaled result >= threshold) is the packed word of columns n0 .. n0+63
      const uint64_t word = __ballot(n < p.N && al * (float)(p.Kreal - 2 * total) >= th);
      if (lane == 0) p.C_bits[m * p.ldc + cb] = word;
    } else if (p.out == kGemmPlanes) {
      const int sv = 2 * total - __builtin_amdgcn_readlane(row_sum, lr);
      if (n < p.N) {
        const int64_t idx = m * p.ldc + lane_off;
        if (p.C_i32) p.C_i32[idx] = sv;
        if (p.C_f32) p.C_f32[idx] = (float)sv / p.levels;
      }
    } else {
      const float ra = CONV ? __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, row_alpha), lr)) : al;
      if (n < p.N) {
        const int64_t idx = m * p.ldc + lane_off;
        const int dot = p.Kreal - 2 * total;
        if (p.out == kGemmI32) p.C_i32[idx] = p.as_count ? p.Kreal - total : dot;
        else if (p.out == kGemmF32) p.C_f32[idx] = (float)dot;
        else p.C_f32[idx] = ra * (float)dot;
      }
    }
  };

  if (S == 1 && p.tail0 >= p.tail1) {
    // one wave holds the whole count of its rows: straight from the accumulators, the
    // planes of one output row (consecutive virtual rows) weighted by their power of two
    int total = 0, pl = 0, lr = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (r < rows_valid) {
        total += acc[r] << pl;
        if (++pl == p.planes) {
          finish(lr++, total);
          total = 0;
          pl = 0;
        }
      }
    }
    return;
  }

  // ---- add the S partial counts of every (row, column) through LDS
  __syncthreads();  // every wave is done with its transposition tile
#pragma unroll
  for (int r = 0; r < R; ++r) lds[(wave * R + r) * 64 + lane] = (uint32_t)acc[r];
  __syncthreads();

  for (int rr = wave; rr < rows_out; rr += S) {
    int total = 0;
    for (int pl = 0; pl < p.planes; ++pl) {
      const int v = rr * p.planes + pl;
      int t = 0;
      // eight independent reads (waves past S repeat the last one and count as zero), so
      // that the LDS round trips overlap instead of adding up
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const int x = (int)lds[((s < S ? s : S - 1) * R + v) * 64 + lane];
        t += (s < S) ? x : 0;
      }
      if (p.tail0 < p.tail1) {
        // K words outside the chunked range (row-major A that may not be read past its
        // last word): plain loads, two dwords per step
        const uint32_t* ar = p.A + (int64_t)(m0 + v) * p.lda;
        const uint32_t* br = p.B + (int64_t)nc * p.ldb;
        for (int d = p.tail0; d < p.tail1; d += 2) {
          const uint2 av = *(const uint2*)(ar + d);
          const uint2 bv = *(const uint2*)(br + d);
          t += __builtin_popcount(OP_AND ? (av.x & bv.x) : (av.x ^ bv.x)) +
               __builtin_popcount(OP_AND ? (av.y & bv.y) : (av.y ^ bv.y));
        }
      }
      total += t << pl;
    }
    finish(rr, total);
  }
}

template <int R, int CH, bool OP_AND, bool PF, bool CONV>
void launch_rs(const GemmParams& p, int S, hipStream_t s) {
  auto kern = gemm_kernel<R, CH, OP_AND, PF, CONV>;
  const int tile_dw = CONV ? 0 : kTileDw;
  const size_t lds_bytes = (size_t)S * (tile_dw > R * 64 ? tile_dw : R * 64) * 4;
  static bool raised = false;  // more than the default 64 KiB of dynamic LDS for S = 8
  if (!raised) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
    raised = true;
  }
  dim3 grid((unsigned)(ceil_div(p.N, 64) * p.row_blocks));
  note_kernel("gemm_kernel<%d,%d,%s,%s,%s> grid %u x %d", R, CH, OP_AND ? "and" : "xor", PF ? "prefetch" : "noprefetch",
              CONV ? "conv" : "gemm", grid.x, 64 * S);
  hipLaunchKernelGGL(kern, grid, dim3(64 * S), lds_bytes, s, p);
}

// Rows per wave and K split.  The kernel runs at full VALU rate once about four waves sit
// on each of the 1024 SIMDs, and its fixed costs (launch, first B chunk, store drain) do not
// shrink with fatter waves, so: the largest R whose grid reaches 4096 waves with a K split
// of at most four.  Larger splits are a last resort: the LDS a workgroup then holds
// (transposition tiles, partial counts) cuts the workgroups per CU, which costs more than
// the extra waves bring.
void choose_shape(const GemmParams& p, bool allow32, int& R_out, int& S_out) {
  const int64_t want = 4096;
  const int smax = p.nch < 8 ? (p.nch > 0 ? p.nch : 1) : 8;
  R_out = 8;
  S_out = smax < 4 ? smax : 4;
  bool found = false;
  // The most rows per wave (fewest loads of the stationary operand) whose grid still reaches
  // the wanted number of waves with a K split of at most four.  Measured per call (operands
  // fresh from the pack kernel), where more waves per block hide the longer first-touch
  // latency: 2048x4096->1024 30.8 us as (32,4) against 32.4 as (8,1); 4096x4096->1024 53.7
  // as (32,2) against 56.4 as (16,1).
  for (int R : {32, 16, 8}) {
    if (R < p.planes || found || (R == 32 && !allow32)) continue;
    const int rpb = (R / p.planes) * p.planes;
    const int64_t blocks = ceil_div(p.N, 64) * ceil_div(p.Mv, rpb);
    const int64_t S = blocks >= want ? 1 : ceil_div(want, blocks);
    if (S <= smax && S <= 4) {
      R_out = R;
      S_out = (int)S;
      found = true;
    }
  }
  if (!found && p.planes <= 8) {  // small problem: 8 rows per wave and as much split as helps
    const int64_t blocks = ceil_div(p.N, 64) * ceil_div(p.Mv, (8 / p.planes) * p.planes);
    const int64_t S = ceil_div(want, blocks);
    S_out = (int)(S < smax ? S : smax);
  }
  if (gemm_tune_rows == 8 || gemm_tune_rows == 16 || (gemm_tune_rows == 32 && allow32)) {
    if (gemm_tune_rows >= p.planes) R_out = gemm_tune_rows;
  }
  if (gemm_tune_ksplit > 0) {
    S_out = gemm_tune_ksplit < 8 ? gemm_tune_ksplit : 8;
    if (S_out > p.nch) S_out = p.nch > 0 ? p.nch : 1;
  }
}

template <bool OP_AND>
void launch(GemmParams& p, hipStream_t s) {
  int R, S;
  choose_shape(p, true, R, S);
  p.rows_per_block = (R / p.planes) * p.planes;
  p.row_blocks = (int)ceil_div(p.Mv, p.rows_per_block);
  p.rows_fastest = gemm_tune_order;
  // (B prefetch registers only where the grid is short of waves anyway: R = 32)
  if (R == 32) launch_rs<32, kChunk, OP_AND, true, false>(p, S, s);
  else if (R == 16) launch_rs<16, kChunk, OP_AND, false, false>(p, S, s);
  else launch_rs<8, kChunk, OP_AND, false, false>(p, S, s);
}

void no_conv(GemmParams& p) {
  p.HoWo = p.Wo = p.Hp = p.Wp_pix = p.Cw = p.stride = p.KWid = 1;
  p.div_howo = p.div_wo = p.div_rw = make_fast_div(1);
}

}  // namespace

hipError_t launch_xnor_gemm(const uint32_t* A, bool a_padded, int64_t lda_dw, const uint64_t* B,
                            int64_t ldb_w, int M, int N, int K, const float* alpha_n, int32_t* C_i32,
                            float* C_f32, uint64_t* C_bits, const float* thr_n, int64_t ldc, hipStream_t s,
                            bool as_count) {
  if ((lda_dw & 1) == 0) {
    hipError_t err = hipSuccess;
    if (launch_xnor_gemm_mfma((const uint64_t*)A, lda_dw / 2, B, ldb_w, M, N, K, alpha_n, C_i32, C_f32,
                              C_bits, thr_n, ldc, s, &err, as_count))
      return err;
  }
  GemmParams p;
  no_conv(p);
  p.A = A;
  p.B = (const uint32_t*)B;
  p.lda = lda_dw;
  p.ldb = ldb_w * 2;
  p.Mv = M;
  p.N = N;
  p.planes = 1;
  p.Kd = (int)(2 * words_for(K));
  p.Kreal = K;
  p.rowsum = nullptr;
  p.alpha = alpha_n;
  p.levels = 1.0f;
  p.C_i32 = C_i32;
  p.C_f32 = C_f32;
  p.C_bits = C_bits;
  p.thr = thr_n;
  p.as_count = as_count ? 1 : 0;
  p.ldc = ldc;
  p.out = C_bits ? kGemmBits : (C_i32 ? kGemmI32 : (alpha_n ? kGemmF32Alpha : kGemmF32));
  if (a_padded) {  // A rows are zero padded to whole chunks: everything runs in the main loop
    p.nch = (int)ceil_div(p.Kd, kChunk);
    p.tail0 = p.tail1 = 0;
  } else {  // whole chunks in the main loop, the remaining words in the epilogue
    p.nch = p.Kd / kChunk;
    p.tail0 = p.nch * kChunk;
    p.tail1 = p.Kd;
  }
  launch<false>(p, s);
  return hipGetLastError();
}

hipError_t launch_plane_gemm(const uint32_t* planes_rows, int64_t lda_dw, int bits,
                             const int32_t* rowsum, const uint64_t* Wb, int64_t ldb_w, int M, int N,
                             int K, int32_t* S, float* out_f32, int64_t ldo, hipStream_t s) {
  if ((lda_dw & 1) == 0) {
    hipError_t err = hipSuccess;
    if (launch_plane_gemm_mfma((const uint64_t*)planes_rows, lda_dw / 2, bits, rowsum, Wb, ldb_w, M, N, K, S,
                               out_f32, ldo, s, &err))
      return err;
  }
  GemmParams p;
  no_conv(p);
  p.A = planes_rows;
  p.B = (const uint32_t*)Wb;
  p.lda = lda_dw;
  p.ldb = ldb_w * 2;
  p.Mv = M * bits;
  p.N = N;
  p.planes = bits;
  p.Kd = (int)(2 * words_for(K));
  p.nch = (int)ceil_div(p.Kd, kChunk);
  p.tail0 = p.tail1 = 0;
  p.Kreal = K;
  p.rowsum = rowsum;
  p.alpha = nullptr;
  p.levels = (float)((1u << bits) - 1u);
  p.C_i32 = S;
  p.C_f32 = out_f32;
  p.C_bits = nullptr;
  p.thr = nullptr;
  p.as_count = 0;
  p.ldc = ldo;
  p.out = kGemmPlanes;
  launch<true>(p, s);
  return hipGetLastError();
}

hipError_t launch_conv_gemm(const uint64_t* Xp, int Nimg, int C, int H, int W, const uint64_t* Wp,
                            int O, int KH, int KW, int stride, int pad, const float* alpha,
                            int32_t* out_i32, float* out_f32, hipStream_t s) {
  const int Ho = (H + 2 * pad - KH) / stride + 1;
  const int Wo = (W + 2 * pad - KW) / stride + 1;
  const int Cw = (int)words_for(C);
  const int kwords = KH * KW * Cw;
  const int ld_words = (int)conv_weight_row_words(kwords);  // row stride
  const int CH = conv_weight_chunk_dwords(kwords);
  GemmParams p;
  p.A = (const uint32_t*)Wp;
  p.B = (const uint32_t*)Xp;
  p.lda = 2 * (int64_t)ld_words;
  p.ldb = 0;
  p.Mv = O;
  p.N = Nimg * Ho * Wo;
  p.planes = 1;
  p.Kd = 2 * kwords;
  p.nch = 2 * (int)conv_weight_bits_words(kwords) / CH;
  p.tail0 = p.tail1 = 0;
  p.Kreal = C * KH * KW;
  p.rowsum = nullptr;
  p.alpha = alpha;
  p.levels = 1.0f;
  p.C_i32 = out_i32;
  p.C_f32 = out_f32;
  p.C_bits = nullptr;
  p.thr = nullptr;
  p.as_count = 0;
  p.ldc = (int64_t)Ho * Wo;
  p.out = out_i32 ? kGemmI32 : (alpha ? kGemmF32Alpha : kGemmF32);
  p.HoWo = Ho * Wo;
  p.Wo = Wo;
  p.Hp = H + 2 * pad;
  p.Wp_pix = W + 2 * pad;
  p.Cw = Cw;
  p.stride = stride;
  p.KWid = KW;
  p.div_howo = make_fast_div((uint32_t)(Ho * Wo));
  p.div_wo = make_fast_div((uint32_t)Wo);
  p.div_rw = make_fast_div((uint32_t)(KW * Cw));
  int R, S;
  choose_shape(p, false, R, S);  // (32 rows per wave measured slower than 16 on every shape)
  p.rows_per_block = R;
  p.row_blocks = (int)ceil_div(p.Mv, R);
  p.rows_fastest = gemm_tune_order;
  if (CH == 32) {
    if (R == 16) launch_rs<16, 32, false, false, true>(p, S, s);
    else launch_rs<8, 32, false, false, true>(p, S, s);
  } else {
    if (R == 16) launch_rs<16, 24, false, false, true>(p, S, s);
    else launch_rs<8, 24, false, false, true>(p, S, s);
  }
  return hipGetLastError();
}

}  // namespace bmx
