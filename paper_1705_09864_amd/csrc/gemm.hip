// xor/and + popcount GEMM on packed operands (VALU integer bound).
// Paper: Sec. 2.2.1 (xnor GEMM on packed words), Sec. 2.2.2 / Eq. 2 (output form), Sec. 2.1
// Eq. 1 for the bit-plane variant.
//
// Shape of the kernel.  C[m][n] = f(sum_k popcount(A[m][k] op B[n][k])).  Lanes span 64
// consecutive columns n (coalesced C rows); a wave owns 8 rows m.  The 8 A rows are the
// same for every lane, so they are streamed through SGPRs with scalar loads and feed
// v_xor_b32 / v_and_b32 as the scalar operand; B rows are staged through LDS in a
// [k-quad][column] layout so that lane n reads its own row 16 bytes at a time without bank
// conflicts.  The inner step is 4 k-dwords x 8 rows = 64 VALU ops against 128 bytes of
// scalar loads and one ds_read_b128.  A workgroup is four waves (32 rows) sharing one B tile.
//
// The scalar side wants whole cache lines per request, so A is read from a row-tiled copy
// At[m/8][k/4][m%8][k%4] (dwords; zero padded in m and k) that the activation pack kernels
// write directly.  bmx_xnor_gemm, whose A arrives row-major and which has no workspace,
// uses the second instantiation that fetches 8 x 16 bytes per step instead.
#include "bmx_internal.h"
#include "scalar_stream.h"

namespace bmx {

namespace {

constexpr int kTileKq = 16;                    // k-quads (of 4 dwords) per LDS tile
constexpr int kLdsCols = 65;                   // 64 columns + 1 pad unit against bank conflicts
constexpr int kTileUnits = kTileKq * kLdsCols;  // 16-byte units per tile buffer

enum GemmOut { kGemmI32 = 0, kGemmF32 = 1, kGemmF32Alpha = 2, kGemmPlanes = 3 };

struct GemmParams {
  const uint32_t* A;      // tiled: At (see above); row-major: [M][lda] dwords
  const uint32_t* B;      // [N][ldb] dwords, K contiguous
  int64_t lda, ldb;       // dwords
  int64_t plane_stride;   // dwords between bit planes of At (planes mode)
  int M, N, Kd;           // Kd = dwords per packed row (even)
  int kq_total;           // k-quads staged through LDS (covers every dword of a row)
  int kq_main;            // k-quads the pipelined loop runs over (== kq_total when tiled)
  int Kreal;              // K in bits (xor modes)
  int planes;             // 1 unless planes mode
  const int32_t* rowsum;  // planes mode: sum_k q[m][k]
  const float* alpha;     // per column n (F32Alpha)
  float levels;           // planes mode: 2^bits - 1
  int32_t* C_i32;
  float* C_f32;
  int64_t ldc;
};

// Eight A rows x four k-dwords in SGPRs.
template <bool TILED>
struct ABlock;

template <>
struct ABlock<true> {  // one contiguous 128-byte record of At
  u32x16 lo, hi;
  __device__ __forceinline__ void issue(const_u32_ptr rec) {
    asm volatile("s_load_dwordx16 %0, %1, 0x0" : "=s"(lo) : "s"(rec));
    asm volatile("s_load_dwordx16 %0, %1, 0x40" : "=s"(hi) : "s"(rec));
  }
  __device__ __forceinline__ void tie() {
    asm volatile("" : "+s"(lo));
    asm volatile("" : "+s"(hi));
  }
  template <int R, int J>
  __device__ __forceinline__ uint32_t get() const {
    if constexpr (R < 4) return lo[R * 4 + J];
    else return hi[(R - 4) * 4 + J];
  }
};

template <>
struct ABlock<false> {  // eight 16-byte pieces, one per row-major A row
  u32x4 r[8];
  __device__ __forceinline__ void issue(const const_u32_ptr* rows, int kq) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      asm volatile("s_load_dwordx4 %0, %1, 0x0" : "=s"(r[i]) : "s"(rows[i] + (int64_t)kq * 4));
  }
  __device__ __forceinline__ void tie() {
#pragma unroll
    for (int i = 0; i < 8; ++i) asm volatile("" : "+s"(r[i]));
  }
  template <int R, int J>
  __device__ __forceinline__ uint32_t get() const {
    return r[R][J];
  }
};

template <bool OP_AND, class AB, int R = 0, int J = 0>
__device__ __forceinline__ void quad_popcount(const AB& a, const uint32_t (&b)[4], int (&pc)[8]) {
  if constexpr (R < 8) {
    const uint32_t av = a.template get<R, J>();
    pc[R] += __builtin_popcount(OP_AND ? (b[J] & av) : (b[J] ^ av));
    asm volatile("" : "+v"(pc[R]));  // keep the op / popcount-accumulate pairs as written
    if constexpr (J < 3) quad_popcount<OP_AND, AB, R, J + 1>(a, b, pc);
    else quad_popcount<OP_AND, AB, R + 1, 0>(a, b, pc);
  }
}

template <bool TILED, bool OP_AND, int OUT>
__global__ void __launch_bounds__(256)
gemm_kernel(const GemmParams p) {
  __shared__ uint4 lds[2][kTileUnits];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = blockIdx.x * 64 + lane;
  const int m0 = (blockIdx.y * 4 + wave) * 8;  // first row of this wave (may be >= M)

  // ---- B tile loader: thread -> (row within 16, k-quad); four passes cover 64 rows
  const int ld_kq = tid & 15;
  const int ld_row = tid >> 4;
  const uint32_t* brow[4];
#pragma unroll
  for (int ps = 0; ps < 4; ++ps) {
    const int row = min(blockIdx.x * 64 + ps * 16 + ld_row, p.N - 1);
    brow[ps] = p.B + (int64_t)row * p.ldb;
  }
  uint2 stage[4][2];
  auto fetch_tile = [&](int tile) {
    const int d0 = (tile * kTileKq + ld_kq) * 4;
    if ((tile + 1) * kTileKq * 4 <= p.Kd) {  // whole tile inside the rows (wave-uniform)
#pragma unroll
      for (int ps = 0; ps < 4; ++ps) {
        stage[ps][0] = *(const uint2*)(brow[ps] + d0);
        stage[ps][1] = *(const uint2*)(brow[ps] + d0 + 2);
      }
    } else {  // last tile: dwords past the row read as zero
#pragma unroll
      for (int ps = 0; ps < 4; ++ps) {
        stage[ps][0] = (d0 < p.Kd) ? *(const uint2*)(brow[ps] + d0) : make_uint2(0, 0);
        stage[ps][1] = (d0 + 2 < p.Kd) ? *(const uint2*)(brow[ps] + d0 + 2) : make_uint2(0, 0);
      }
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int ps = 0; ps < 4; ++ps)
      lds[buf][ld_kq * kLdsCols + ps * 16 + ld_row] =
          make_uint4(stage[ps][0].x, stage[ps][0].y, stage[ps][1].x, stage[ps][1].y);
  };

  // ---- A stream (wave-uniform)
  const int m8 = min(m0 / 8, (p.M - 1) / 8);  // waves past the last row block repeat it
  const_u32_ptr arows[8];
  if constexpr (!TILED) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
      arows[i] = (const_u32_ptr)uniform_addr((uint64_t)(uintptr_t)p.A +
                                             (int64_t)min(m8 * 8 + i, p.M - 1) * p.lda * 4);
  }

  int acc[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) acc[r] = 0;
  const int ntiles = (p.kq_total + kTileKq - 1) / kTileKq;

  for (int plane = 0; plane < p.planes; ++plane) {
    const_u32_ptr arec = (const_u32_ptr)uniform_addr(
        (uint64_t)(uintptr_t)p.A + ((int64_t)plane * p.plane_stride + (int64_t)m8 * p.kq_total * 32) * 4);
    int pc[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      pc[r] = 0;
      asm volatile("" : "+v"(pc[r]));
    }
    ABlock<TILED> ab[2];
    if (p.kq_main > 0) {
      if constexpr (TILED) ab[0].issue(arec);
      else ab[0].issue(arows, 0);
    }
    int kq_next = 1;  // global k-quad the next issue fetches

    fetch_tile(0);  // (the barrier closing the previous plane's last tile protects buffer 0)
    store_tile(0);
    __syncthreads();

    for (int tile = 0; tile < ntiles; ++tile) {
      const int buf = tile & 1;
      const int nkq = min(kTileKq, p.kq_main - tile * kTileKq);
      if (tile + 1 < ntiles) fetch_tile(tile + 1);
      uint4 bv[2];
      bv[0] = lds[buf][lane];
      for (int s = 0; s < nkq; s += 2) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          if (h == 1 && s + 1 >= nkq) break;  // odd tail (row-major A only), wave-uniform
          const uint32_t b[4] = {bv[h].x, bv[h].y, bv[h].z, bv[h].w};
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          ab[h].tie();
          // request the next A block and the next B quad, then work on the current ones
          asm volatile("" : "+v"(pc[0]));
          const int kqn = min(kq_next, p.kq_main - 1);
          if constexpr (TILED) ab[h ^ 1].issue(arec + (int64_t)kqn * 32);
          else ab[h ^ 1].issue(arows, kqn);
          kq_next += 1;
          asm volatile("" : "+v"(pc[0]));
          bv[h ^ 1] = lds[buf][min(s + h + 1, nkq - 1) * kLdsCols + lane];
          quad_popcount<OP_AND>(ab[h], b, pc);
        }
      }
      if (tile + 1 < ntiles) store_tile(buf ^ 1);
      __syncthreads();
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if constexpr (!TILED) {
      if (p.Kd & 2) {
        // Row-major A with a trailing half quad: two dwords per row, fetched exactly (a
        // 16-byte piece would run past the row) against the B quad still held in LDS.
        const int kq = p.Kd / 4;
        const uint4 bq = lds[(kq / kTileKq) & 1][(kq % kTileKq) * kLdsCols + lane];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const uint32_t a0 = arows[i][kq * 4], a1 = arows[i][kq * 4 + 1];
          pc[i] += __builtin_popcount(OP_AND ? (bq.x & a0) : (bq.x ^ a0)) +
                   __builtin_popcount(OP_AND ? (bq.y & a1) : (bq.y ^ a1));
        }
      }
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) acc[r] += pc[r] << plane;
  }

  // ---- epilogue: lanes write 64 consecutive columns of each of the wave's rows
  if (n < p.N) {
    float al = 1.0f;
    if (OUT == kGemmF32Alpha) al = p.alpha[n];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int m = m0 + r;
      if (m < p.M) {
        const int64_t idx = (int64_t)m * p.ldc + n;
        if (OUT == kGemmPlanes) {
          const int sv = 2 * acc[r] - p.rowsum[m];
          if (p.C_i32) p.C_i32[idx] = sv;
          if (p.C_f32) p.C_f32[idx] = (float)sv / p.levels;
        } else {
          const int dot = p.Kreal - 2 * acc[r];
          if (OUT == kGemmI32) p.C_i32[idx] = dot;
          else if (OUT == kGemmF32) p.C_f32[idx] = (float)dot;
          else p.C_f32[idx] = al * (float)dot;
        }
      }
    }
  }
}

template <bool TILED, bool OP_AND, int OUT>
void launch(const GemmParams& p, hipStream_t s) {
  dim3 grid((unsigned)ceil_div(p.N, 64), (unsigned)ceil_div(p.M, 32));
  hipLaunchKernelGGL((gemm_kernel<TILED, OP_AND, OUT>), grid, dim3(256), 0, s, p);
}

}  // namespace

hipError_t launch_xnor_gemm(const uint32_t* A, bool a_tiled, int64_t lda_dw, const uint64_t* B,
                            int64_t ldb_w, int M, int N, int K, const float* alpha_n, int32_t* C_i32,
                            float* C_f32, int64_t ldc, hipStream_t s) {
  GemmParams p;
  p.A = A;
  p.B = (const uint32_t*)B;
  p.lda = lda_dw;
  p.ldb = ldb_w * 2;
  p.plane_stride = 0;
  p.M = M;
  p.N = N;
  p.Kd = (int)(2 * words_for(K));
  p.Kreal = K;
  p.planes = 1;
  p.rowsum = nullptr;
  p.alpha = alpha_n;
  p.levels = 1.0f;
  p.C_i32 = C_i32;
  p.C_f32 = C_f32;
  p.ldc = ldc;
  if (a_tiled) {
    p.kq_total = p.kq_main = (int)tiled_kq(K);
    if (C_i32) launch<true, false, kGemmI32>(p, s);
    else if (alpha_n) launch<true, false, kGemmF32Alpha>(p, s);
    else launch<true, false, kGemmF32>(p, s);
  } else {
    // whole k-quads in the pipelined loop; a trailing half quad gets its own exact step
    p.kq_total = (p.Kd + 3) / 4;
    p.kq_main = p.Kd / 4;
    if (C_i32) launch<false, false, kGemmI32>(p, s);
    else if (alpha_n) launch<false, false, kGemmF32Alpha>(p, s);
    else launch<false, false, kGemmF32>(p, s);
  }
  return hipGetLastError();
}

hipError_t launch_plane_gemm(const uint32_t* planes_tiled, int bits, const int32_t* rowsum,
                             const uint64_t* Wb, int M, int N, int K, int32_t* S, float* out_f32,
                             int64_t ldo, hipStream_t s) {
  GemmParams p;
  p.A = planes_tiled;
  p.B = (const uint32_t*)Wb;
  p.lda = 0;
  p.ldb = 2 * words_for(K);
  p.plane_stride = tiled_bytes(M, K) / 4;
  p.M = M;
  p.N = N;
  p.Kd = (int)(2 * words_for(K));
  p.kq_total = p.kq_main = (int)tiled_kq(K);
  p.Kreal = K;
  p.planes = bits;
  p.rowsum = rowsum;
  p.alpha = nullptr;
  p.levels = (float)((1u << bits) - 1u);
  p.C_i32 = S;
  p.C_f32 = out_f32;
  p.ldc = ldo;
  launch<true, true, kGemmPlanes>(p, s);
  return hipGetLastError();
}

}  // namespace bmx
