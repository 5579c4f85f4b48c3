// fp32 GEMM for the fp32 workload (tiny, launch-latency bound): C[M,N] = sum_k A(m,k) * B(n,k) with
// the same layouts and epilogues as the bf16 kernel (Sec. 2.2: Y = X W^T, dX = dY W, dW += dY^T X).
// Plain LDS-tiled FMA kernel: 64 x 64 tile, 256 threads, 4 x 4 outputs per thread, any M/N/K.
#include "common.h"

namespace {

template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                       float* __restrict__ C, const float* __restrict__ R, int M, int N,
                                                       int K, long sam, long sak, long sbn, long sbk, int ldc) {
  constexpr int T = 64, KT = 16;
  __shared__ float As[KT][T + 4];
  __shared__ float Bs[KT][T + 4];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * T, n0 = blockIdx.x * T;
  const int ty = tid >> 4, tx = tid & 15;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += KT) {
    for (int e = tid; e < T * KT; e += 256) {
      int r, k;
      if (sak == 1) { r = e / KT; k = e % KT; } else { r = e % T; k = e / T; }   // walk the contiguous index fastest
      int gm = m0 + r, gk = k0 + k;
      As[k][r] = (gm < M && gk < K) ? A[gm * sam + gk * sak] : 0.f;
    }
    for (int e = tid; e < T * KT; e += 256) {
      int r, k;
      if (sbk == 1) { r = e / KT; k = e % KT; } else { r = e % T; k = e / T; }
      int gn = n0 + r, gk = k0 + k;
      Bs[k][r] = (gn < N && gk < K) ? B[gn * sbn + gk * sbk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < KT; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
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
      size_t off = (size_t)m * ldc + n;
      float v = acc[i][j];
      if (EPI == EPI_RESID) v += R[off];
      if (EPI == EPI_ACCUM) v += C[off];
      C[off] = v;
    }
  }
}

}  // namespace

hipError_t launch_gemm_f32(int layout, int epi, const void* A, const void* B, void* C, const void* R, int M, int N,
                           int K, int lda, int ldb, int ldc, hipStream_t s) {
  if (M <= 0 || N <= 0 || K <= 0) return hipErrorInvalidValue;
  long sam, sak, sbn, sbk;
  if (layout == GEMM_NT) { sam = lda; sak = 1; sbn = ldb; sbk = 1; }
  else if (layout == GEMM_TN) { sam = 1; sak = lda; sbn = 1; sbk = ldb; }
  else return hipErrorInvalidValue;
  dim3 grid((N + 63) / 64, (M + 63) / 64), block(256);
  const float *a = (const float*)A, *b = (const float*)B, *r = (const float*)R;
  float* c = (float*)C;
  if (epi == EPI_STORE || epi == EPI_STOREF) hipLaunchKernelGGL(gemm_f32_kernel<EPI_STORE>, grid, block, 0, s, a, b, c, r,
      M, N, K, sam, sak, sbn, sbk, ldc);
  else if (epi == EPI_RESID) hipLaunchKernelGGL(gemm_f32_kernel<EPI_RESID>, grid, block, 0, s, a, b, c, r, M, N, K, sam, sak, sbn, sbk, ldc);
  else if (epi == EPI_ACCUM) hipLaunchKernelGGL(gemm_f32_kernel<EPI_ACCUM>, grid, block, 0, s, a, b, c, r, M, N, K, sam, sak, sbn, sbk, ldc);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}
