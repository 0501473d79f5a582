// fp32 debug path: plain LDS-tiled fp32 FMA kernels, no matrix cores, every intermediate in fp32.
// It exists to validate the boundary, the input generators and the oracle plumbing independently of
// the bf16 kernels, and serves the single factored linear layer O = (X U) V (paper Sec. 4.2.1).
#include "common.h"

namespace svdmlp {

constexpr int TM = 64, TN = 64, TK = 16;

// C[M,N] = A[M,K] B[K,N]           (GATED == false)
// C[M,N] = SiLU(A B) .* (A2 B2)    (GATED == true; epilogue of paper Alg. 3)
// Row-major with leading dimensions lda / ldb / ldc.  256 threads, each a 4x4 micro-tile.
// Partial sums of each 16-wide k tile are formed separately and then added to the running total,
// which keeps the fp32 rounding error of long contractions (K = ffn) well below 1e-6 relative.
template <bool GATED>
__global__ __launch_bounds__(256) void k_f32_gemm(const float* __restrict__ A, int lda, const float* __restrict__ B, int ldb,
                                                  const float* __restrict__ A2, const float* __restrict__ B2,
                                                  float* __restrict__ C, int ldc, int M, int N, int K) {
  __shared__ float sA[TK][TM + 1], sB[TK][TN];
  __shared__ float sA2[GATED ? TK : 1][TM + 1], sB2[GATED ? TK : 1][TN];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  float acc[4][4] = {}, acc2[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += TK) {
    for (int i = threadIdx.x; i < TM * TK; i += 256) {
      int mm = i / TK, kk = i % TK;
      int m = m0 + mm, k = k0 + kk;
      bool ok = m < M && k < K;
      sA[kk][mm] = ok ? A[(size_t)m * lda + k] : 0.f;
      if (GATED) sA2[kk][mm] = ok ? A2[(size_t)m * lda + k] : 0.f;
    }
    for (int i = threadIdx.x; i < TK * TN; i += 256) {
      int kk = i / TN, nn = i % TN;
      int k = k0 + kk, n = n0 + nn;
      bool ok = k < K && n < N;
      sB[kk][nn] = ok ? B[(size_t)k * ldb + n] : 0.f;
      if (GATED) sB2[kk][nn] = ok ? B2[(size_t)k * ldb + n] : 0.f;
    }
    __syncthreads();
    float part[4][4] = {}, part2[4][4] = {};
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = sA[kk][ty * 4 + i]; b[i] = sB[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) part[i][j] = fmaf(a[i], b[j], part[i][j]);
      if (GATED) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { a[i] = sA2[kk][ty * 4 + i]; b[i] = sB2[kk][tx * 4 + i]; }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) part2[i][j] = fmaf(a[i], b[j], part2[i][j]);
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) { acc[i][j] += part[i][j]; if (GATED) acc2[i][j] += part2[i][j]; }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[i][j];
      if (GATED) v = v / (1.0f + expf(-v)) * acc2[i][j];
      C[(size_t)m * ldc + n] = v;
    }
  }
}

static int gemm(bool gated, const float* A, int lda, const float* B, int ldb, const float* A2, const float* B2, float* C,
                int ldc, int64_t M, int64_t N, int64_t K, hipStream_t st) {
  dim3 grid((unsigned)((N + TN - 1) / TN), (unsigned)((M + TM - 1) / TM));
  if (gated)
    hipLaunchKernelGGL(k_f32_gemm<true>, grid, dim3(256), 0, st, A, lda, B, ldb, A2, B2, C, ldc, (int)M, (int)N, (int)K);
  else
    hipLaunchKernelGGL(k_f32_gemm<false>, grid, dim3(256), 0, st, A, lda, B, ldb, A2, B2, C, ldc, (int)M, (int)N, (int)K);
  return (int)hipGetLastError();
}

int f32_forward(const Ctx* c, const void* Xv, int64_t M, void* Yv, hipStream_t st) {
  const Plan& p = c->plan;
  const svdmlp_desc& de = c->desc;
  const float* X = static_cast<const float*>(Xv);
  float* Y = static_cast<float*>(Yv);
  float* ws = reinterpret_cast<float*>(c->ws);
  const int d = (int)p.d, ffn = (int)p.ffn, r = (int)p.r, rd = (int)p.rd;
  int e;
  if (p.kind == SVDMLP_LINEAR) {
    float* T = ws + p.f32_T;
    if ((e = gemm(false, X, d, (const float*)de.Ug, r, nullptr, nullptr, T, r, M, r, d, st))) return e;
    return gemm(false, T, r, (const float*)de.Vg, ffn, nullptr, nullptr, Y, ffn, M, ffn, r, st);
  }
  float* T = ws + p.f32_T;    // [M, 2r]: gate strip in columns [0,r), up strip in [r,2r)
  float* H = ws + p.f32_H;    // [M, ffn]
  float* Td = ws + p.f32_Td;  // [M, rd]
  if ((e = gemm(false, X, d, (const float*)de.Ug, r, nullptr, nullptr, T, 2 * r, M, r, d, st))) return e;
  if ((e = gemm(false, X, d, (const float*)de.Uu, r, nullptr, nullptr, T + r, 2 * r, M, r, d, st))) return e;
  if ((e = gemm(true, T, 2 * r, (const float*)de.Vg, ffn, T + r, (const float*)de.Vu, H, ffn, M, ffn, r, st))) return e;
  if ((e = gemm(false, H, ffn, (const float*)de.Ud, rd, nullptr, nullptr, Td, rd, M, rd, ffn, st))) return e;
  return gemm(false, Td, rd, (const float*)de.Vd, d, nullptr, nullptr, Y, d, M, d, rd, st);
}

}  // namespace svdmlp
