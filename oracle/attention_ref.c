/* Eq. 1 of ASPD Sec. 3.2 with an explicit dense mask (Eq. 2-3), float64, plain loops.
 *
 * TEST INFRASTRUCTURE (see oracle/__init__.py): a second, independent writing of oracle/attention.py's
 * attend_queries, with no library routine underneath (no BLAS), parallelised over (query row, query head)
 * with OpenMP so that it can be timed on all host cores next to the GPU numbers.  No tiling, no running
 * softmax, no split of the key range: per (row, head) the scores over ALL slots are formed, masked keys
 * get no weight, one softmax is taken.
 *
 *   q    [n][Hq][D]    queries
 *   k, v [T][Hkv][D]   the sequence's rows in slot order (gathered by the caller)
 *   mask [n][T]        1 = visible (Eq. 2: M = 0), 0 = not (M = -inf); every row has a visible key
 *   out  [n][Hq][D],  lse [n][Hq] = max + log(sum exp)
 * Query head h reads KV head h / (Hq / Hkv).  Returns the number of OpenMP threads used.
 */
#include <math.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int aspd_oracle_attend(const double* q, const double* k, const double* v, const unsigned char* mask, int n, int T,
                       int Hq, int Hkv, int D, double scale, double* out, double* lse) {
  const int G = Hq / Hkv;
  int threads = 1;
#ifdef _OPENMP
  threads = omp_get_max_threads();
#endif
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
#pragma omp for collapse(2) schedule(dynamic, 1)
    for (int r = 0; r < n; ++r) {
      for (int h = 0; h < Hq; ++h) {
        const double* qr = q + ((size_t)r * Hq + h) * D;
        const int kh = h / G;
        double m = -INFINITY;
        for (int j = 0; j < T; ++j) {
          if (!mask[(size_t)r * T + j]) continue;
          const double* kr = k + ((size_t)j * Hkv + kh) * D;
          double dot = 0.0;
          for (int d = 0; d < D; ++d) dot += qr[d] * kr[d];
          s[j] = dot * scale;
          if (s[j] > m) m = s[j];
        }
        double denom = 0.0;
        double* o = out + ((size_t)r * Hq + h) * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        for (int j = 0; j < T; ++j) {
          if (!mask[(size_t)r * T + j]) continue;
          const double p = exp(s[j] - m);
          denom += p;
          const double* vr = v + ((size_t)j * Hkv + kh) * D;
          for (int d = 0; d < D; ++d) o[d] += p * vr[d];
        }
        for (int d = 0; d < D; ++d) o[d] /= denom;
        lse[(size_t)r * Hq + h] = m + log(denom);
      }
    }
    free(s);
  }
  return threads;
}
