/* Naive masked triple loop for O = W_s x I.  TEST INFRASTRUCTURE ONLY.
 *
 * Section 5 ("GPU Implementation") defines the operation as the product of the
 * sparse weight matrix with the dense activation matrix; written out it is
 *     O[m][n] = sum_k mask[m][k] * W[m][k] * I[k][n].
 * The mask is the dense M x K 0/1 matrix (the Kronecker product of the factor
 * matrices, built by the Python side of the oracle); no adjacency lists, no
 * tiling, no reordering: k ascends, n is innermost, accumulation in double.
 * With take_abs != 0 the same loop sums |W|*|I| (the denominator of the
 * parity tests' error metric).  OpenMP splits rows m over the host cores; the
 * sum for each output is formed by one thread in a fixed order.
 *
 * Shares no code with the HIP library.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int rbgp_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void rbgp_oracle_spmm(const uint8_t *mask, const float *W, const float *I,
                      double *O, long M, long K, long N, int take_abs) {
#pragma omp parallel for schedule(static)
  for (long m = 0; m < M; ++m) {
    double *acc = O + m * N;
    memset(acc, 0, (size_t)N * sizeof(double));
    for (long k = 0; k < K; ++k) {
      if (!mask[m * K + k]) continue;
      double w = (double)W[m * K + k];
      const float *row = I + k * N;
      if (take_abs) {
        w = fabs(w);
        for (long n = 0; n < N; ++n) acc[n] += w * fabs((double)row[n]);
      } else {
        for (long n = 0; n < N; ++n) acc[n] += w * (double)row[n];
      }
    }
  }
}
