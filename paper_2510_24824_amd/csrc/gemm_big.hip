// bf16 projections with many rows (prefill: M = sequences x positions): c = a[M,K] * w[N,K]^T on
// gfx950 matrix cores, MFMA-bound.  Workgroup tile 256 rows x 256 columns, K in slices of 64 through
// LDS with the next slice prefetched into registers; 8 waves as 2 x 4, each 128 rows x 64 columns =
// 8 x 4 tiles of v_mfma_f32_16x16x32_bf16 (weights = A operand, activations = B operand: a lane ends
// up with 4 consecutive columns of one row).  The wave tile is what bounds this kernel: every MFMA
// needs 0.375 KB of LDS fragment reads (0.5 KB with 64 x 64 wave tiles, which ran LDS-bound).
// Two epilogues:
//   EPI_F32    : float c[M,N]                                        (QKV, output, down projections)
//   EPI_SWIGLU : w = [W_gate; W_up] ([2F,K]); the tile holds 128 gate columns and the matching 128 up
//                columns and writes silu(gate) * up as bf16 act[M,F]              (SwiGLU, fused)
#include "plt_internal.h"

namespace plt {

typedef __attribute__((ext_vector_type(4))) float f32x4;

namespace {

constexpr int GB_BM = 256, GB_BN = 256, GB_BK = 64, GB_LDK = GB_BK + 8, GB_THREADS = 512;
constexpr int GB_HALF = GB_BN / 2;   // SwiGLU tile: GB_HALF gate columns + the matching GB_HALF up columns
enum { EPI_F32 = 0, EPI_SWIGLU = 1 };

template <int EPI>
__global__ __launch_bounds__(GB_THREADS) void k_gemm_big(const bf16_t* __restrict__ a, const bf16_t* __restrict__ w,
                                                         void* __restrict__ out, int M, int N, int K) {
  // N: EPI_F32: output columns (= rows of w); EPI_SWIGLU: F (w has 2F rows, the output F columns)
  __shared__ __attribute__((aligned(16))) bf16_t As[GB_BM * GB_LDK];
  __shared__ __attribute__((aligned(16))) bf16_t Ws[GB_BN * GB_LDK];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, m16 = lane & 15, g = lane >> 4;
  const int wm = wv >> 2, wn = wv & 3;
  const int m0 = blockIdx.y * GB_BM;
  const int n0 = blockIdx.x * (EPI == EPI_SWIGLU ? GB_HALF : GB_BN);
  // global row of w behind local tile row r
  auto wrow = [&](int r) -> int {
    if (EPI == EPI_SWIGLU) { const int c = n0 + (r & (GB_HALF - 1)); return c < N ? (r < GB_HALF ? c : N + c) : -1; }
    const int c = n0 + r; return c < N ? c : -1;
  };
  uint4 ra[4], rw[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { ra[i] = make_uint4(0, 0, 0, 0); rw[i] = make_uint4(0, 0, 0, 0); }
  const int ks_total = K / GB_BK;

  f32x4 acc[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int ks = -1; ks < ks_total; ++ks) {
    if (ks >= 0) {
      __syncthreads();                 // previous slice consumed
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ch = tid + i * GB_THREADS, row = ch >> 3, kc = (ch & 7) * 8;
        *reinterpret_cast<uint4*>(&As[row * GB_LDK + kc]) = ra[i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ch = tid + i * GB_THREADS, row = ch >> 3, kc = (ch & 7) * 8;
        *reinterpret_cast<uint4*>(&Ws[row * GB_LDK + kc]) = rw[i];
      }
      __syncthreads();
    }
    if (ks + 1 < ks_total) {           // prefetch slice ks + 1 into registers
      const int k0 = (ks + 1) * GB_BK;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ch = tid + i * GB_THREADS, row = ch >> 3, kc = (ch & 7) * 8;
        const int gm = m0 + row;
        ra[i] = gm < M ? *reinterpret_cast<const uint4*>(a + (size_t)gm * K + k0 + kc) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int ch = tid + i * GB_THREADS, row = ch >> 3, kc = (ch & 7) * 8;
        const int gr = wrow(row);
        rw[i] = gr >= 0 ? *reinterpret_cast<const uint4*>(w + (size_t)gr * K + k0 + kc) : make_uint4(0, 0, 0, 0);
      }
    }
    if (ks < 0) continue;
#pragma unroll
    for (int k32 = 0; k32 < GB_BK / 32; ++k32) {
      uint4 fw[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        // EPI_SWIGLU: tiles 0,1 = this wave's 32 gate columns, tiles 2,3 = the matching up columns
        const int r = EPI == EPI_SWIGLU ? (j < 2 ? wn * 32 + j * 16 : GB_HALF + wn * 32 + (j - 2) * 16) : wn * 64 + j * 16;
        fw[j] = *reinterpret_cast<const uint4*>(&Ws[(r + m16) * GB_LDK + k32 * 32 + g * 8]);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint4 fa = *reinterpret_cast<const uint4*>(&As[(wm * 128 + i * 16 + m16) * GB_LDK + k32 * 32 + g * 8]);
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fw[j]),
                                                             __builtin_bit_cast(bf16x8, fa), acc[i][j], 0, 0, 0);
      }
    }
  }
  // acc[i][j][e]: row m0 + wm*128 + i*16 + m16, column (tile j) + 4*g + e
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int gm = m0 + wm * 128 + i * 16 + m16;
    if (gm >= M) continue;
    if (EPI == EPI_SWIGLU) {
      bf16_t* o = (bf16_t*)out + (size_t)gm * N;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int gn = n0 + wn * 32 + j * 16 + 4 * g;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) { const float gt = acc[i][j][e]; v[e] = gt / (1.0f + __expf(-gt)) * acc[i][j + 2][e]; }
        if (gn + 3 < N && (N & 3) == 0) {
          ushort4 p; p.x = f32_to_bf16(v[0]); p.y = f32_to_bf16(v[1]); p.z = f32_to_bf16(v[2]); p.w = f32_to_bf16(v[3]);
          *reinterpret_cast<ushort4*>(o + gn) = p;
        } else {
          for (int e = 0; e < 4; ++e) if (gn + e < N) o[gn + e] = f32_to_bf16(v[e]);
        }
      }
    } else {
      float* o = (float*)out + (size_t)gm * N;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int gn = n0 + wn * 64 + j * 16 + 4 * g;
        if (gn + 3 < N && (N & 3) == 0) *reinterpret_cast<f32x4*>(o + gn) = acc[i][j];
        else for (int e = 0; e < 4; ++e) if (gn + e < N) o[gn + e] = acc[i][j][e];
      }
    }
  }
}

}  // namespace

// Worth it only when the 256 x 256 tiles still fill the chip (prefill-sized row counts); decode-sized
// launches with a few hundred rows keep the small-tile split-K kernel.
bool gemm_big_applies(int M, int N, int K) {
  const long tiles = (long)((M + GB_BM - 1) / GB_BM) * ((N + GB_BN - 1) / GB_BN);
  return M >= 512 && tiles >= 200 && (K % GB_BK) == 0;
}

void launch_gemm_big(hipStream_t s, const bf16_t* a, const bf16_t* w, float* c, int M, int N, int K) {
  dim3 grid((N + GB_BN - 1) / GB_BN, (M + GB_BM - 1) / GB_BM);
  hipLaunchKernelGGL(k_gemm_big<EPI_F32>, grid, dim3(GB_THREADS), 0, s, a, w, (void*)c, M, N, K);
}

void launch_gemm_big_swiglu(hipStream_t s, const bf16_t* a, const bf16_t* wgu, bf16_t* act, int M, int F, int K) {
  dim3 grid((F + GB_HALF - 1) / GB_HALF, (M + GB_BM - 1) / GB_BM);
  hipLaunchKernelGGL(k_gemm_big<EPI_SWIGLU>, grid, dim3(GB_THREADS), 0, s, a, wgu, (void*)act, M, F, K);
}

}  // namespace plt
