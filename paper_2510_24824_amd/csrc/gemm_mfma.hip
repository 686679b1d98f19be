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

// ----------------------------------------------------------------------------------------------
// Weight-streaming variant for few rows (M <= 128 per row block), weights read once.  It served every decode
// projection until the row tiles of gemm_big.hip overtook it (rows_split_applies below); it remains the kernel for
// few-row products with K below 1024, K no multiple of 64, or fewer than 256 columns.
//
// A workgroup owns one K range of KR = 512 and keeps the matching slice of the activations
// (up to 128 rows x 512, bf16) resident in LDS.  Its 4 waves (one per SIMD, so each may use the
// whole register file) walk over groups of NB 16-column strips of the weight matrix: the strips'
// rows go from HBM straight into registers in MFMA A-operand layout (16 bytes per lane), half a
// K range at a time, the next half prefetched while the current one is multiplied; the
// activations come from LDS as the B operand and every fragment read from LDS feeds NB MFMAs
// (LDS bandwidth, not HBM, bounds this kernel when NB is small).  No barrier after the prologue.
// Each K range writes its own float slab; consumers add the slabs in a fixed order.
namespace plt {

constexpr int WS_KR = 512, WS_LDK = WS_KR + 8;

// MT: 16-row activation tiles (4: M <= 64, 8: M <= 128); NB: strips per group; the K range is
// consumed in steps of WS_KH 32-wide chunks, two register buffers alternating
template <int MT, int NB, int NW>   // NW: waves per workgroup (4: one per SIMD, 8: two per SIMD)
__global__ __launch_bounds__(NW * 64) void k_gemm_wstream(const bf16_t* __restrict__ a, const bf16_t* __restrict__ w,
                                                             float* __restrict__ c, int M, int N, int K,
                                                             int n_groups) {
  extern __shared__ __attribute__((aligned(16))) bf16_t As[];   // [MT*16][WS_LDK]
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, m16 = lane & 15, g = lane >> 4;
  const int ng = blockIdx.x, rb = blockIdx.y, split = blockIdx.z;
  const int row0 = rb * (MT * 16);
  const int range0 = split;                    // this workgroup's K range (slab = blockIdx.z)

  constexpr int WS_THREADS = NW * 64;
  constexpr int WS_KH = (NB * NW >= 16) ? 4 : 8, STEPS = (WS_KR / 32) / WS_KH;
  const int n_strips = (N + 15) >> 4;
  const int n_grp = (n_strips + NB - 1) / NB;
  const int stride = n_groups * NW;
  uint4 bufA[NB][WS_KH], bufB[NB][WS_KH];
  // step h (0..STEPS-1) of K range `rng` for the NB strips of group grp
  auto wload = [&](uint4 (&f)[NB][WS_KH], int grp, int h, int rng) {
    const int k0 = rng * WS_KR;
    const int kr = (K - k0 < WS_KR) ? K - k0 : WS_KR;          // valid width of this K range
#pragma unroll
    for (int sb = 0; sb < NB; ++sb) {
      int n = (grp * NB + sb) * 16 + m16; if (n >= N) n = N - 1;   // ragged N: clamp (stores are masked)
      const bf16_t* wr = w + (size_t)n * K + k0 + g * 8;
#pragma unroll
      for (int kk = 0; kk < WS_KH; ++kk) {
        int ko = (h * WS_KH + kk) * 32; if (ko + g * 8 + 8 > kr) ko = 0;   // beyond K: in-range chunk (meets zeros)
        f[sb][kk] = *reinterpret_cast<const uint4*>(wr + ko);
      }
    }
  };
  // Activation slice of K range `rng` -> LDS.  A full range goes HBM/L2 -> LDS directly, one row (1 KB) per
  // wavefront load, no registers involved (rows beyond M repeat row M-1; their outputs are never stored).
  // The ragged last range of a K that is no multiple of 512 is staged through registers in small batches
  // so that the columns beyond K can be zero-filled.
  const unsigned lds_as = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)As;
  auto load_slice = [&](int rng) {
    const int k0 = rng * WS_KR;
    const int kr = (K - k0 < WS_KR) ? K - k0 : WS_KR;
    if (kr == WS_KR) {
#pragma unroll 4
      for (int row = wv; row < MT * 16; row += NW) {
        int gm = row0 + row; if (gm >= M) gm = M - 1;
        const bf16_t* src = a + (size_t)gm * K + k0 + lane * 8;
        const unsigned dst = __builtin_amdgcn_readfirstlane(lds_as + (unsigned)row * (WS_LDK * 2));
        unsigned keep_m0;                                          // m0 is left as it was found
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                     : "=&s"(keep_m0) : "s"(dst), "v"(src) : "memory");
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      return;
    }
    constexpr int TOTAL = MT * 16 * (WS_KR / 8) / WS_THREADS;   // 16-byte chunks per thread
    constexpr int BATCH = 8;
#pragma unroll 1
    for (int b0 = 0; b0 < TOTAL; b0 += BATCH) {
      uint4 v[BATCH];
#pragma unroll
      for (int it = 0; it < BATCH; ++it) {
        const int ch = tid + (b0 + it) * WS_THREADS;
        const int row = ch / (WS_KR / 8), kc = (ch % (WS_KR / 8)) * 8;
        v[it] = make_uint4(0, 0, 0, 0);
        if (row0 + row < M && kc < kr) v[it] = *reinterpret_cast<const uint4*>(a + (size_t)(row0 + row) * K + k0 + kc);
      }
#pragma unroll
      for (int it = 0; it < BATCH; ++it) {
        const int ch = tid + (b0 + it) * WS_THREADS;
        const int row = ch / (WS_KR / 8), kc = (ch % (WS_KR / 8)) * 8;
        *reinterpret_cast<uint4*>(&As[row * WS_LDK + kc]) = v[it];
      }
    }
  };
  // the first weight fragments are requested before the prologue so that their latency hides behind it
  int grp = ng * NW + wv;
  if (grp < n_grp) wload(bufA, grp, 0, range0);
  load_slice(range0);
  __syncthreads();

  f32x4 acc[NB][MT];
  auto mac = [&](const uint4 (&f)[NB][WS_KH], int h) {
#pragma unroll
    for (int kk = 0; kk < WS_KH; ++kk) {
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const uint4 af = *reinterpret_cast<const uint4*>(&As[(i * 16 + m16) * WS_LDK + (h * WS_KH + kk) * 32 + g * 8]);
#pragma unroll
        for (int sb = 0; sb < NB; ++sb)
          acc[sb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f[sb][kk]),
                                                              __builtin_bit_cast(bf16x8, af), acc[sb][i], 0, 0, 0);
      }
      // keep the LDS reads of later K chunks from being hoisted up here (register pressure)
      if ((kk & 1) == 1) __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto zero_acc = [&]() {
#pragma unroll
    for (int sb = 0; sb < NB; ++sb)
#pragma unroll
      for (int i = 0; i < MT; ++i) acc[sb][i] = f32x4{0.f, 0.f, 0.f, 0.f};
  };
  float* cs = c + (size_t)split * M * N;
  auto store_acc = [&](int gq) {
    // acc[sb][i][e] = C[row0 + i*16 + m16][(gq*NB + sb)*16 + 4*g + e]
#pragma unroll
    for (int sb = 0; sb < NB; ++sb) {
      const int gn = (gq * NB + sb) * 16 + 4 * g;
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int gm = row0 + i * 16 + m16;
        if (gm >= M || gn >= N) continue;
        float* dst = cs + (size_t)gm * N + gn;
        if (gn + 3 < N && (N & 3) == 0) *reinterpret_cast<f32x4*>(dst) = acc[sb][i];
        else for (int e = 0; e < 4; ++e) if (gn + e < N) dst[e] = acc[sb][i][e];
      }
    }
  };
  for (; grp < n_grp; grp += stride) {
    zero_acc();
#pragma unroll
    for (int t = 0; t < STEPS; ++t) {            // STEPS is even: buffer parity carries over to the next group
      if (t + 1 < STEPS) { if (t & 1) wload(bufA, grp, t + 1, range0); else wload(bufB, grp, t + 1, range0); }
      else if (grp + stride < n_grp) wload(bufA, grp + stride, 0, range0);
      if (t & 1) mac(bufB, t); else mac(bufA, t);
    }
    store_acc(grp);
  }
}

bool gemm_use_wstream(int M, int N, int K) { return M <= 256 && N >= 16; }

// Launch shape of the streaming kernel.  One workgroup fits per compute unit (its activation slice fills
// most of the LDS), so at most 256 workgroups: a second round would pay the prologue again.  Strips per
// wave task (NB) grow until the NW * n_groups waves of one (K range, row block) cover the strips in one pass
// if possible.  (Letting a workgroup walk 2 or 4 K ranges with the accumulators kept in registers halves
// or removes the split-K slabs; measured inside the decode step it was slower than one range per workgroup.)
struct WsPlan { int S, rbs, n_groups, nb; bool small; };
static WsPlan ws_plan(int M, int N, int K) {
  WsPlan p;
  const int NWv = 4;
  p.S = (K + WS_KR - 1) / WS_KR;
  p.small = M <= 64;
  p.rbs = p.small ? 1 : (M + 127) / 128;
  const int n_strips = (N + 15) / 16;
  int n_groups = 256 / (p.S * p.rbs); if (n_groups < 1) n_groups = 1;
  const int slots = n_groups * NWv;
  int nb = (n_strips + slots - 1) / slots;
  nb = nb >= 3 ? 4 : (nb == 2 ? 2 : 1);
  const int n_grp = (n_strips + nb - 1) / nb;
  if (n_groups > (n_grp + NWv - 1) / NWv) n_groups = (n_grp + NWv - 1) / NWv;
  p.n_groups = n_groups; p.nb = nb;
  return p;
}

// Decode-sized projections (up to 1024 rows, K from 1024 on) run as row tiles of the tile kernel with K split over
// about 256 workgroups: 64 / 128 / 256 rows x 64 columns x a run of K slices, three or four LDS stages, one float slab
// per K run (one slab, i.e. whole K, when the tiles alone fill the chip: wide projections from 257 rows on).  Measured
// in the decode step against the streaming kernel above: batch 64 L = 1 / 2 / 3 / 4 -1.8 / -3.0 / -3.2 / -2.3 %, batch 1
// -7.9 %, batch 16 -5.6 % (fewer and smaller slabs: 8 runs of K for the down projection instead of 11 ranges, and what
// a kernel leaves dirty in eight L2s is drained at its boundary).  The streaming kernel keeps short K and tiny N.
static bool rows_split_applies(int M, int N, int K) {
  return M >= 1 && M <= 1024 && N >= 256 && K >= 1024 && (K % 64) == 0 && !gemm_big_applies(M, N, K);
}
// splits for the generic entry: the streaming kernel writes one slab per workgroup K span
int gemm_bf16_splits_any(int M, int N, int K) {
  if (rows_split_applies(M, N, K)) return gemm_rows_split_slabs(M, N, K);
  if (gemm_use_wstream(M, N, K)) return ws_plan(M, N, K).S;
  if (gemm_big_applies(M, N, K)) return 1;
  return gemm_bf16_splits(M, N, K);
}

template <int MT, int NB, int NW>
static void ws_launch(hipStream_t s, const bf16_t* a, const bf16_t* w, float* c, int M, int N, int K, const WsPlan& p) {
  const size_t lds = (size_t)MT * 16 * WS_LDK * sizeof(bf16_t);
  // opt-in to more than 64 KB of dynamic LDS: once per template instance, thread-safe (initialisation of a local static)
  static const hipError_t attr_once = hipFuncSetAttribute((const void*)k_gemm_wstream<MT, NB, NW>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  (void)attr_once;
  hipLaunchKernelGGL((k_gemm_wstream<MT, NB, NW>), dim3(p.n_groups, p.rbs, p.S), dim3(NW * 64), lds, s, a, w, c, M, N, K,
                     p.n_groups);
}

void launch_gemm_bf16_any(hipStream_t s, const bf16_t* a, const bf16_t* w, float* c, int M, int N, int K) {
  if (rows_split_applies(M, N, K)) { launch_gemm_rows_split(s, a, w, c, M, N, K); return; }
  if (!gemm_use_wstream(M, N, K)) {
    if (gemm_big_applies(M, N, K)) launch_gemm_big(s, a, w, c, M, N, K);
    else launch_gemm_bf16(s, a, w, c, M, N, K, gemm_bf16_splits(M, N, K));
    return;
  }
  // 4 waves (one per SIMD) or 8: measured equal within noise on the decode shapes; 4 is used
  const WsPlan p = ws_plan(M, N, K);
#define WS_CASE(MT_, NB_) ws_launch<MT_, NB_, 4>(s, a, w, c, M, N, K, p)
  if (p.small) { if (p.nb == 4) WS_CASE(4, 4); else if (p.nb == 2) WS_CASE(4, 2); else WS_CASE(4, 1); }
  else         { if (p.nb == 4) WS_CASE(8, 4); else if (p.nb == 2) WS_CASE(8, 2); else WS_CASE(8, 1); }
#undef WS_CASE
}

}  // namespace plt
