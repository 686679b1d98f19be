// bf16 projections on gfx950 matrix cores: c[M,N] (float) = a[M,K] * w[N,K]^T.
//
// Every projection of block f (QKV [Alg. 3 l.1], output [Alg. 3 l.6], SwiGLU up/gate and
// down, classifier head) is this contraction.  While decoding, M = batch x L rows is small
// (128..1024) and the weights are read once per step for all L loop stages -- the saving
// cross-loop parallelism buys over L serial passes [Sec. 2.2.1].
//
// Tiling: workgroup = 128 rows x 64 columns, K in slices of 64 through LDS (register
// prefetch of the next slice); 4 waves as 2 x 2, each wave 64 rows x 32 columns =
// 4 x 2 tiles of v_mfma_f32_16x16x32_bf16.  The weight rows are the MFMA A operand and the
// activation rows the B operand, so a lane ends up with 4 consecutive output columns of one
// row (one 16-byte store).  Optional split-K writes one float slab per split; the consumer
// kernel sums the slabs in a fixed order (deterministic, no atomics).
#include "plt_internal.h"

namespace plt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int BM = 128, BN = 64, BK = 64, LDK = BK + 8;   // LDS row stride 144 B: conflict-light

__global__ __launch_bounds__(256) void k_gemm_bf16(const bf16_t* __restrict__ a, const bf16_t* __restrict__ w,
                                                   float* __restrict__ c, int M, int N, int K,
                                                   int ksteps_per_split) {
  __shared__ __attribute__((aligned(16))) bf16_t As[BM * LDK];
  __shared__ __attribute__((aligned(16))) bf16_t Ws[BN * LDK];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, m16 = lane & 15, g = lane >> 4;
  const int wm = wv >> 1, wn = wv & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN, split = blockIdx.z;
  const int ks_total = K / BK;
  const int ks_beg = split * ksteps_per_split;
  int ks_end = ks_beg + ksteps_per_split; if (ks_end > ks_total) ks_end = ks_total;

  // global -> register staging: A tile 128x64 = 1024 chunks of 8 elements (4 per thread),
  // W tile 64x64 = 512 chunks (2 per thread); chunk c -> row c/8, k-offset (c%8)*8
  uint4 ra[4], rw[2];
  auto gload = [&](int ks) {
    const int k0 = ks * BK;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int ch = tid + i * 256, row = ch >> 3, kc = (ch & 7) * 8;
      const int gm = m0 + row;
      ra[i] = gm < M ? *reinterpret_cast<const uint4*>(a + (size_t)gm * K + k0 + kc) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int ch = tid + i * 256, row = ch >> 3, kc = (ch & 7) * 8;
      const int gn = n0 + row;
      rw[i] = gn < N ? *reinterpret_cast<const uint4*>(w + (size_t)gn * K + k0 + kc) : make_uint4(0, 0, 0, 0);
    }
  };
  auto sstore = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int ch = tid + i * 256, row = ch >> 3, kc = (ch & 7) * 8;
      *reinterpret_cast<uint4*>(&As[row * LDK + kc]) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int ch = tid + i * 256, row = ch >> 3, kc = (ch & 7) * 8;
      *reinterpret_cast<uint4*>(&Ws[row * LDK + kc]) = rw[i];
    }
  };

  f32x4 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  if (ks_beg < ks_end) gload(ks_beg);
  for (int ks = ks_beg; ks < ks_end; ++ks) {
    __syncthreads();                 // LDS free (previous slice consumed)
    sstore();
    __syncthreads();
    if (ks + 1 < ks_end) gload(ks + 1);
#pragma unroll
    for (int k32 = 0; k32 < BK / 32; ++k32) {
      uint4 fa[4], fw[2];
#pragma unroll
      for (int i = 0; i < 4; ++i)
        fa[i] = *reinterpret_cast<const uint4*>(&As[(wm * 64 + i * 16 + m16) * LDK + k32 * 32 + g * 8]);
#pragma unroll
      for (int j = 0; j < 2; ++j)
        fw[j] = *reinterpret_cast<const uint4*>(&Ws[(wn * 32 + j * 16 + m16) * LDK + k32 * 32 + g * 8]);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
              __builtin_bit_cast(bf16x8, fw[j]), __builtin_bit_cast(bf16x8, fa[i]), acc[i][j], 0, 0, 0);
    }
  }
  // acc[i][j][e] = C[row = m0 + wm*64 + i*16 + m16][col = n0 + wn*32 + j*16 + 4*g + e]
  float* cs = c + (size_t)split * M * N;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + wm * 64 + i * 16 + m16;
    if (gm >= M) continue;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int gn = n0 + wn * 32 + j * 16 + 4 * g;
      float* dst = cs + (size_t)gm * N + gn;
      if (gn + 3 < N && (N & 3) == 0) {
        *reinterpret_cast<f32x4*>(dst) = acc[i][j];
      } else {
        for (int e = 0; e < 4; ++e) if (gn + e < N) dst[e] = acc[i][j][e];
      }
    }
  }
}

// Number of K splits: enough workgroups to cover the 256 compute units when M x N alone gives
// few tiles, bounded so that every split keeps at least 4 K-slices.
int gemm_bf16_splits(int M, int N, int K) {
  const long tiles = (long)((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const int ks_total = K / BK;
  int s = (int)((256 + tiles - 1) / tiles);
  int cap = ks_total / 4; if (cap < 1) cap = 1;
  if (s > cap) s = cap;
  if (s > 16) s = 16;
  if (s < 1) s = 1;
  return s;
}

void launch_gemm_bf16(hipStream_t s, const bf16_t* a, const bf16_t* w, float* c, int M, int N, int K,
                      int splits) {
  const int ks_total = K / BK;
  const int per = (ks_total + splits - 1) / splits;
  dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM, splits);
  hipLaunchKernelGGL(k_gemm_bf16, grid, dim3(256), 0, s, a, w, c, M, N, K, per);
}

}  // namespace plt
