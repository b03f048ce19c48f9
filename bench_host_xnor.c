/* Host-side xnor GEMM on 64-bit packed words: the method of the paper's Sec. 2.2.1 (xnor +
 * popcount over BINARY_WORDs, its xnor_64_omp variant: 64-bit words, OpenMP over the output)
 * timed on the benchmark host's own cores, so that the paper's CPU speed-ups (Sec. 3.1) have a
 * like-for-like neighbour next to the GPU figures.
 *
 * CONTEXT FOR bench.py ONLY.  It is not the oracle (that is the float layer under oracle/), it
 * checks nothing, and nothing in the library or the tests links it.  bench.py compiles it with
 * the host compiler when it runs.
 *
 *   A [M][Kw], B [N][Kw] uint64 words packed along K, tail bits zero in both;
 *   C[m][n] = K - 2 * sum_w popcount(A[m][w] ^ B[n][w])   (= 2 * xnor_count - K, Eq. 2).
 *
 * Loop structure: output rows are shared out over the threads; a thread walks its row of A
 * against four rows of B at a time, so that each word of A loaded serves four counts. */
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int host_xnor_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void host_xnor_gemm(const uint64_t* A, const uint64_t* B, int32_t* C, long M, long N, long Kw, long K,
                    int threads) {
#ifdef _OPENMP
  if (threads > 0) omp_set_num_threads(threads);
#endif
#pragma omp parallel for schedule(static)
  for (long m = 0; m < M; ++m) {
    const uint64_t* a = A + m * Kw;
    long n = 0;
    for (; n + 4 <= N; n += 4) {
      const uint64_t *b0 = B + n * Kw, *b1 = b0 + Kw, *b2 = b1 + Kw, *b3 = b2 + Kw;
      long c0 = 0, c1 = 0, c2 = 0, c3 = 0;
      for (long w = 0; w < Kw; ++w) {
        const uint64_t av = a[w];
        c0 += __builtin_popcountll(av ^ b0[w]);
        c1 += __builtin_popcountll(av ^ b1[w]);
        c2 += __builtin_popcountll(av ^ b2[w]);
        c3 += __builtin_popcountll(av ^ b3[w]);
      }
      C[m * N + n] = (int32_t)(K - 2 * c0);
      C[m * N + n + 1] = (int32_t)(K - 2 * c1);
      C[m * N + n + 2] = (int32_t)(K - 2 * c2);
      C[m * N + n + 3] = (int32_t)(K - 2 * c3);
    }
    for (; n < N; ++n) {
      const uint64_t* b = B + n * Kw;
      long c = 0;
      for (long w = 0; w < Kw; ++w) c += __builtin_popcountll(a[w] ^ b[w]);
      C[m * N + n] = (int32_t)(K - 2 * c);
    }
  }
}
