/*
 * fp64 CPU oracle for the SVD-factored MLP forward.  TEST INFRASTRUCTURE ONLY:
 * it exists so the GPU library can be checked against something written from
 * the paper alone.  It shares no code with the HIP path and must never be
 * called from it.
 *
 * What it computes is not an approximation: the method re-associates a chain
 * of matrix products, so the oracle is that chain written out with plain
 * loops, IEEE double throughout, no intermediate rounding, no blocking, no
 * fusion.
 *
 *   low-rank linear (paper Sec. 3.1, "XW -> XUV"; Eq. 1 is its block form):
 *       T[m,p] = sum_k X[m,k] U[k,p]            O[m,n] = sum_p T[m,p] V[p,n]
 *
 *   gated MLP (paper Sec. 4.2.2 and Alg. 2 / Alg. 3: gate and up projections,
 *   SiLU on the gate branch, element-wise product, down projection; argument
 *   shapes follow the "Require" line of Alg. 2, r2 being the down rank):
 *       Tg = X Ug          Tu = X Uu                     [M, r]
 *       G  = Tg Vg         P  = Tu Vu                    [M, N]
 *       H  = SiLU(G) .* P,  SiLU(x) = x / (1 + exp(-x))  (Alg. 3, epilogue)
 *       Td = H Ud                                         [M, r2]
 *       Z  = Td Vd                                        [M, K]
 *
 * The paper never defines SiLU; the standard x*sigmoid(x) is used.  No bias
 * terms appear anywhere in Alg. 2 / Alg. 3, so none are applied.
 *
 * All matrices are dense row-major doubles.  Rows of X are independent, so the
 * only parallelism is an OpenMP loop over rows; summation inside a row is
 * plain left to right in index order.
 *
 * Pins (tests/test_oracle_pins.py): full-rank factors from an exact SVD give
 * X W to 1e-10; the rank-r truncation error equals the root sum of squares of
 * the dropped singular values (Eckart-Young); brute-force dense evaluation on
 * tiny integer inputs; special cases (zero gate factor, identity factors,
 * linearity of the up branch); numpy float64 matmul chains on random inputs.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* out[n] += a * row[n], n < N  (the inner, contiguous loop of an i-k-j product) */
static void axpy_row(double a, const double *row, double *out, int64_t N) {
  for (int64_t n = 0; n < N; ++n) out[n] += a * row[n];
}

/* out[0..N) = sum_k x[k] * W[k, 0..N),  W row-major [K, N] */
static void row_times_matrix(const double *x, const double *W, int64_t K, int64_t N, double *out) {
  for (int64_t n = 0; n < N; ++n) out[n] = 0.0;
  for (int64_t k = 0; k < K; ++k) axpy_row(x[k], W + k * N, out, N);
}

double svdmlp_oracle_silu(double x) { return x / (1.0 + exp(-x)); }

int svdmlp_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* O = (X U) V.  X[M,K], U[K,r], V[r,N], O[M,N].  Returns 0, or -1 on bad args / OOM. */
int svdmlp_oracle_linear(const double *X, int64_t M, int64_t K, int64_t N, int64_t r,
                         const double *U, const double *V, double *O) {
  if (!X || !U || !V || !O || M < 0 || K <= 0 || N <= 0 || r <= 0) return -1;
  int fail = 0;
#pragma omp parallel
  {
    double *T = (double *)malloc(sizeof(double) * (size_t)r);
    if (!T) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
      if (!T) continue;
      row_times_matrix(X + m * K, U, K, r, T);
      row_times_matrix(T, V, r, N, O + m * N);
    }
    free(T);
  }
  return fail ? -1 : 0;
}

/*
 * Z = ((SiLU((X Ug) Vg) .* ((X Uu) Vu)) Ud) Vd.
 * X[M,K], Ug/Uu[K,r], Vg/Vu[r,N], Ud[N,r2], Vd[r2,K], Z[M,K].
 * H_out (may be NULL) receives the N-wide activation H[M,N] for inspection.
 */
int svdmlp_oracle_gated(const double *X, int64_t M, int64_t K, int64_t N, int64_t r, int64_t r2,
                        const double *Ug, const double *Vg, const double *Uu, const double *Vu,
                        const double *Ud, const double *Vd, double *Z, double *H_out) {
  if (!X || !Ug || !Vg || !Uu || !Vu || !Ud || !Vd || !Z) return -1;
  if (M < 0 || K <= 0 || N <= 0 || r <= 0 || r2 <= 0) return -1;
  int fail = 0;
#pragma omp parallel
  {
    double *Tg = (double *)malloc(sizeof(double) * (size_t)r);
    double *Tu = (double *)malloc(sizeof(double) * (size_t)r);
    double *G = (double *)malloc(sizeof(double) * (size_t)N);
    double *P = (double *)malloc(sizeof(double) * (size_t)N);
    double *Td = (double *)malloc(sizeof(double) * (size_t)r2);
    int ok = Tg && Tu && G && P && Td;
    if (!ok) {
#pragma omp atomic write
      fail = 1;
    }
#pragma omp for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
      if (!ok) continue;
      const double *x = X + m * K;
      row_times_matrix(x, Ug, K, r, Tg);
      row_times_matrix(x, Uu, K, r, Tu);
      row_times_matrix(Tg, Vg, r, N, G);
      row_times_matrix(Tu, Vu, r, N, P);
      for (int64_t n = 0; n < N; ++n) G[n] = svdmlp_oracle_silu(G[n]) * P[n]; /* G now holds H */
      if (H_out) memcpy(H_out + m * N, G, sizeof(double) * (size_t)N);
      row_times_matrix(G, Ud, N, r2, Td);
      row_times_matrix(Td, Vd, r2, K, Z + m * K);
    }
    free(Tg); free(Tu); free(G); free(P); free(Td);
  }
  return fail ? -1 : 0;
}
