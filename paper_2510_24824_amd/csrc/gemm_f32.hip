// float GEMM for the PLT_F32 configuration (tiny models; parity at 1e-5 needs true float
// products, so no bf16 MFMA here).  c[M,N] = a[M,K] * w[N,K]^T, 64x64 tile per workgroup,
// K staged through LDS in slices of 16, each thread owns a 4x4 patch.  Any M, N, K.
#include "plt_internal.h"

namespace plt {

__global__ __launch_bounds__(256) void k_gemm_f32(const float* __restrict__ a, const float* __restrict__ w,
                                                  float* __restrict__ c, int M, int N, int K) {
  __shared__ float As[16][64 + 4];
  __shared__ float Ws[16][64 + 4];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    // 64 rows x 16 k = 1024 elements per operand, 4 per thread; k fastest in memory
    for (int e = threadIdx.x; e < 1024; e += 256) {
      int row = e >> 4, kk = e & 15;
      int gm = m0 + row, gn = n0 + row, gk = k0 + kk;
      As[kk][row] = (gm < M && gk < K) ? a[(size_t)gm * K + gk] : 0.f;
      Ws[kk][row] = (gn < N && gk < K) ? w[(size_t)gn * K + gk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float av[4], wv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = As[kk][ty * 4 + i]; wv[i] = Ws[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], wv[j], acc[i][j]);
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i) {
    int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
    for (int j = 0; j < 4; ++j) {
      int gn = n0 + tx * 4 + j;
      if (gn < N) c[(size_t)gm * N + gn] = acc[i][j];
    }
  }
}

void launch_gemm_f32(hipStream_t s, const float* a, const float* w, float* c, int M, int N, int K) {
  hipLaunchKernelGGL(k_gemm_f32, dim3((N + 63) / 64, (M + 63) / 64), dim3(256), 0, s, a, w, c, M, N, K);
}

}  // namespace plt
