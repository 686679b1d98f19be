// Tiled bf16 projections c = a[M,K] * w[N,K]^T on gfx950 matrix cores, whole K per workgroup (no split-K).
// Prefill (M = sequences x positions, MFMA-bound): workgroup tile 256 rows x 256 columns, K in slices of 64
// through LDS, loaded HBM -> LDS directly and two slices deep; 8 waves as 2 x 4, each 128 rows x 64 columns =
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

constexpr int GB_BK = 64;
enum { EPI_F32 = 0, EPI_SWIGLU = 1 };

// Operand tiles go HBM -> LDS directly (global_load_lds, 16 bytes per lane, no register staging), two
// stages deep, one barrier per K slice.  A tile row holds 64 K-values = 8 chunks of 16 bytes; chunk kc of
// row r sits in slot r*8 + (kc ^ (r & 7)): the direct load writes lane l of a wave to consecutive slots,
// so each lane simply fetches the chunk that belongs in its slot, and the XOR makes the fragment reads
// (16 rows x one chunk column per quarter wave) touch every bank once.
//
// BM x BN: workgroup tile; WM x WN waves, each (BM/WM) x (BN/WN).  Instances:
//   256 x 256, 2 x 4 waves of 128 x 64 : prefill-sized row counts (MFMA-bound).  Two waves along N (128 x 128
//       per wave, accumulators in AGPRs, one wave per SIMD) halve the LDS reads per MFMA but measured 1.5x
//       slower: a single wave per SIMD cannot hide the LDS and barrier latency.
//   256 x 64, 4 x 2 waves of 64 x 32 : the gate/up projection of decode steps with 129..256 rows, SwiGLU fused
//       (all rows of the step in one tile, whole K: no split-K slabs, no separate activation kernel).  The same
//       tile for the plain QKV projection measured slower than the weight-streaming kernel and is not used.
template <int EPI, int BM, int BN, int WM, int WN, int STAGES = 2>
__global__ __launch_bounds__(WM * WN * 64) void k_gemm_tile(const bf16_t* __restrict__ a, const bf16_t* __restrict__ w,
                                                          void* __restrict__ out, int M, int N, int K) {
  // N: EPI_F32: output columns (= rows of w); EPI_SWIGLU: F (w has 2F rows, the output F columns)
  constexpr int THREADS = WM * WN * 64;
  constexpr int MI = BM / WM / 16, NT = BN / WN / 16;       // 16 x 16 tiles per wave: rows, columns
  constexpr int DMA_A = BM * GB_BK / 8 / THREADS, DMA_W = BN * GB_BK / 8 / THREADS;   // 16-byte chunks per thread
  constexpr int HALF = BN / 2;                              // SwiGLU tile: HALF gate columns + the matching HALF up columns
  constexpr int A_BYTES = BM * GB_BK * 2, W_BYTES = BN * GB_BK * 2, STAGE_BYTES = A_BYTES + W_BYTES;
  static_assert(DMA_A >= 1 && DMA_W >= 1 && (EPI != EPI_SWIGLU || NT % 2 == 0), "tile shape");
  extern __shared__ __attribute__((aligned(16))) char gb_lds[];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, m16 = lane & 15, g = lane >> 4;
  const int wm = wv / WN, wn = wv % WN;
  const int m0 = blockIdx.y * BM;
  const int n0 = blockIdx.x * (EPI == EPI_SWIGLU ? HALF : BN);
  const int w_rows = EPI == EPI_SWIGLU ? 2 * N : N;
  // global row of w behind local tile row r (rows beyond the matrix: clamped, their outputs are never stored)
  auto wrow = [&](int r) -> int {
    int gr;
    if (EPI == EPI_SWIGLU) { const int c = n0 + (r & (HALF - 1)); gr = r < HALF ? c : N + c; if (c >= N) gr = w_rows - 1; }
    else { gr = n0 + r; }
    return gr < w_rows ? gr : w_rows - 1;
  };
  // this thread's chunks of the A tile and of the W tile: slot s = i*THREADS + tid -> row s/8, chunk (s%8) ^ (row%8)
  const bf16_t* pa[DMA_A]; const bf16_t* pw[DMA_W];
#pragma unroll
  for (int i = 0; i < DMA_A; ++i) {
    const int sl = i * THREADS + tid, row = sl >> 3, kc = (sl & 7) ^ (row & 7);
    int gm = m0 + row; if (gm >= M) gm = M - 1;
    pa[i] = a + (size_t)gm * K + kc * 8;
  }
#pragma unroll
  for (int i = 0; i < DMA_W; ++i) {
    const int sl = i * THREADS + tid, row = sl >> 3, kc = (sl & 7) ^ (row & 7);
    pw[i] = w + (size_t)wrow(row) * K + kc * 8;
  }
  // Direct load issued as an instruction of its own (not through the compiler's builtin): the compiler
  // orders every later LDS read after a builtin direct load (it cannot tell the two stages apart), which
  // would serialise load and compute.  Here the only wait is the explicit one in front of the barrier.
  const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)gb_lds;
  auto dma16 = [](const bf16_t* src, unsigned lds_wave_base) {   // lane l: 16 bytes -> LDS[lds_wave_base + 16 l]
    unsigned keep_m0;                                            // m0 is left as it was found
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep_m0) : "s"(lds_wave_base), "v"(src) : "memory");
  };
  auto issue = [&](int ks) {
    const unsigned stage = lds0 + (unsigned)(ks % STAGES) * STAGE_BYTES;
    const int k0 = ks * GB_BK;
#pragma unroll
    for (int i = 0; i < DMA_A; ++i)
      dma16(pa[i] + k0, stage + __builtin_amdgcn_readfirstlane((unsigned)(i * THREADS + wv * 64) * 16));
#pragma unroll
    for (int i = 0; i < DMA_W; ++i)
      dma16(pw[i] + k0, stage + A_BYTES + __builtin_amdgcn_readfirstlane((unsigned)(i * THREADS + wv * 64) * 16));
  };
  const int ks_total = K / GB_BK;

  f32x4 acc[MI][NT];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  // fragment addressing: row r = (multiple of 16) + m16, chunk kc = k32*4 + g -> slot r*8 + (kc ^ (m16 & 7))
  const int sw0 = (g ^ (m16 & 7)) * 16;                 // byte offset of the lane's chunk inside its row, k32 = 0
  // STAGES - 1 slices are requested ahead: with two stages a slice has one K step to arrive (enough when the matrix
  // cores are the limit, as in prefill); the decode-row tile is latency-bound with that (a slice of 40 KB per round
  // trip), so it runs three stages and waits only for the OLDEST slice in flight (loads return in order)
#pragma unroll
  for (int st = 0; st < STAGES - 1; ++st) if (st < ks_total) issue(st);
  for (int ks = 0; ks < ks_total; ++ks) {
    // this wave's part of slice ks has landed: everything but the (STAGES - 2) younger slices still in flight
    if (STAGES == 2 || ks + STAGES - 2 >= ks_total) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(%0)" :: "n"((STAGES - 2) * (DMA_A + DMA_W)) : "memory");
    // ... and everyone's; every wave is done with slice ks - 1, whose stage is refilled next.  With more than two
    // stages the bare barrier instruction: __syncthreads() would drain the younger slices too (its fence waits for
    // every load in flight); the asm statements on both sides keep the LDS reads where they are
    if (STAGES == 2) __syncthreads(); else __builtin_amdgcn_s_barrier();
    if (ks + STAGES - 1 < ks_total) issue(ks + STAGES - 1);
    else asm volatile("" ::: "memory");
    const char* As = gb_lds + (ks % STAGES) * STAGE_BYTES;
    const char* Ws = As + A_BYTES;
#pragma unroll
    for (int k32 = 0; k32 < GB_BK / 32; ++k32) {
      const int sw = sw0 ^ (k32 * 64);                  // chunk index ^ 4
      uint4 fw[NT];
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        // EPI_SWIGLU: the first half of the tiles = this wave's gate columns, the second half = the matching up columns
        const int r = EPI == EPI_SWIGLU ? (j < NT / 2 ? wn * (NT * 8) + j * 16 : HALF + wn * (NT * 8) + (j - NT / 2) * 16)
                                        : wn * (NT * 16) + j * 16;
        fw[j] = *reinterpret_cast<const uint4*>(Ws + (r + m16) * 128 + sw);
      }
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const uint4 fa = *reinterpret_cast<const uint4*>(As + (wm * (MI * 16) + i * 16 + m16) * 128 + sw);
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fw[j]),
                                                             __builtin_bit_cast(bf16x8, fa), acc[i][j], 0, 0, 0);
      }
    }
  }
  // acc[i][j][e]: row m0 + wm*MI*16 + i*16 + m16, column (tile j) + 4*g + e
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int gm = m0 + wm * (MI * 16) + i * 16 + m16;
    if (gm >= M) continue;
    if (EPI == EPI_SWIGLU) {
      bf16_t* o = (bf16_t*)out + (size_t)gm * N;
#pragma unroll
      for (int j = 0; j < NT / 2; ++j) {
        const int gn = n0 + wn * (NT * 8) + j * 16 + 4 * g;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) { const float gt = acc[i][j][e]; v[e] = gt * __builtin_amdgcn_rcpf(1.0f + __expf(-gt)) * acc[i][j + NT / 2][e]; }   // 1-ulp reciprocal: the result is rounded to bf16
        if (gn + 3 < N && (N & 3) == 0) {
          const f32x4 vv = {v[0], v[1], v[2], v[3]};               // hardware conversion (nearest even), two instructions
          *reinterpret_cast<bf16x4*>(o + gn) = __builtin_convertvector(vv, bf16x4);
        } else {
          for (int e = 0; e < 4; ++e) if (gn + e < N) o[gn + e] = f32_to_bf16(v[e]);
        }
      }
    } else {
      float* o = (float*)out + (size_t)gm * N;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int gn = n0 + wn * (NT * 16) + j * 16 + 4 * g;
        if (gn + 3 < N && (N & 3) == 0) *reinterpret_cast<f32x4*>(o + gn) = acc[i][j];
        else for (int e = 0; e < 4; ++e) if (gn + e < N) o[gn + e] = acc[i][j][e];
      }
    }
  }
}

template <int EPI, int BM, int BN, int WM, int WN, int STAGES = 2>
void tile_launch(hipStream_t s, const bf16_t* a, const bf16_t* w, void* out, int M, int N, int K) {
  constexpr int LDS_BYTES = STAGES * (BM + BN) * GB_BK * 2;     // stages x (A tile + W tile)
  // opt-in to more than 64 KB of dynamic LDS: once per template instance, thread-safe (initialisation of a local static)
  static const hipError_t attr_once = hipFuncSetAttribute((const void*)k_gemm_tile<EPI, BM, BN, WM, WN, STAGES>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  (void)attr_once;
  const int ncols = EPI == EPI_SWIGLU ? BN / 2 : BN;             // output columns per tile
  dim3 grid((N + ncols - 1) / ncols, (M + BM - 1) / BM);
  hipLaunchKernelGGL((k_gemm_tile<EPI, BM, BN, WM, WN, STAGES>), grid, dim3(WM * WN * 64), LDS_BYTES, s, a, w, out, M, N, K);
}

}  // namespace

// Worth it only when the 256 x 256 tiles still fill the chip (prefill-sized row counts); decode-sized
// launches with a few hundred rows keep the weight-streaming kernel.
bool gemm_big_applies(int M, int N, int K) {
  const long tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
  return M >= 512 && tiles >= 200 && (K % GB_BK) == 0;
}

void launch_gemm_big(hipStream_t s, const bf16_t* a, const bf16_t* w, float* c, int M, int N, int K) {
  tile_launch<EPI_F32, 256, 256, 2, 4>(s, a, w, (void*)c, M, N, K);
}

void launch_gemm_big_swiglu(hipStream_t s, const bf16_t* a, const bf16_t* wgu, bf16_t* act, int M, int F, int K) {
  tile_launch<EPI_SWIGLU, 256, 256, 2, 4>(s, a, wgu, (void*)act, M, F, K);
}

// Decode step: act[M, F] = silu(a Wg^T) * (a Wu^T) for up to 256 rows in one launch, no slabs.
// Measured inside the decode step: at 129..256 rows (where the streaming kernel needs two row blocks and
// its slabs double) this is 5 % of the step faster; up to 128 rows the streaming kernel plus the separate
// activation kernel is as fast or faster, so those row counts keep it.
bool gemm_swiglu_rows_applies(int M, int F, int K) {
  return M > 128 && M <= 256 && (K % GB_BK) == 0 && (F + 31) / 32 >= 128;   // enough 32-column tiles to occupy the chip
}

// the same tile with the plain float epilogue: wide projections at 129..256 rows, whole K, no slabs
void launch_gemm_rows_tile(hipStream_t s, const bf16_t* a, const bf16_t* w, float* c, int M, int N, int K) {
  tile_launch<EPI_F32, 256, 64, 4, 2, 3>(s, a, w, (void*)c, M, N, K);
}

void launch_gemm_swiglu_rows(hipStream_t s, const bf16_t* a, const bf16_t* wgu, bf16_t* act, int M, int F, int K) {
  tile_launch<EPI_SWIGLU, 256, 64, 4, 2, 3>(s, a, wgu, (void*)act, M, F, K);
}

}  // namespace plt
