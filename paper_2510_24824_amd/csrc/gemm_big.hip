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
//   EPI_RESID  : float c[M,N] += product (the residual stream updated in place by the output / down projection)
//   EPI_ROPE_DEC : the same for the rows of a decode step (64 rows x 128 columns per workgroup, a wave = 16 rows x one
//                or two whole heads); row (b, l) appends to the shared cache (l = 0) or to ring l - 1 [Alg. 1 l.5-7]
//   EPI_ROPE   : w = W_qkv of a prefill chunk; waves as 4 x 2 so that a wave holds whole heads (64 rows x 128
//                columns): rotary embedding, gate logit and the cache appends straight from the accumulators
//                [Alg. 3 l.1, l.4; Sec. 2.2.2] - the float QKV matrix is never written
#include "plt_internal.h"
#include "rope_epilogue.h"

namespace plt {

namespace {

constexpr int GB_BK = 64;
enum { EPI_F32 = 0, EPI_SWIGLU = 1, EPI_ROPE = 2, EPI_RESID = 3, EPI_ROPE_DEC = 4 };

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
//   256 / 128 / 64 x 64, waves of 64 x 32 (32 x 32 for the 64-row tile) : the gate/up projection of decode steps,
//       SwiGLU fused (all rows of the step in one tile, whole K: no split-K slabs, no separate activation kernel),
//       three LDS stages (four for the 64-row tile).  The plain projections of decode steps run on the same tiles
//       with K split into runs over gridDim.z (one float slab per run).
template <int EPI, int BM, int BN, int WM, int WN, int STAGES = 2, int D = 128, typename KT = bf16_t>
__global__ __launch_bounds__(WM * WN * 64) void k_gemm_tile(const bf16_t* __restrict__ a, const bf16_t* __restrict__ w,
                                                          void* __restrict__ out, int M, int N, int K, const RopeEpi ep) {
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
  int tile_m = blockIdx.y, tile_n = blockIdx.x;
  if constexpr (BM == 256 && BN == 256) {
    // Prefill tiles: which tile a workgroup takes follows the dies.  Workgroups go to the 8 dies round-robin in launch
    // order, and a die's cache (4 MB) only helps tiles that run on it AT THE SAME TIME (a tile streams 2 MB of
    // operands per 2048 of K): so die x takes a contiguous run of the tile sequence in which 32 consecutive tiles are
    // 8 row tiles x 4 column tiles (12 operand panels for 32 tiles instead of ~17 in launch order).
    constexpr int NXCD = 8, PR = 8;
    const int TM = gridDim.y, TN = gridDim.x, total = TM * TN;
    const int bid = blockIdx.y * TN + blockIdx.x, x = bid % NXCD, q = bid / NXCD;
    const int v = x * (total / NXCD) + min(x, total % NXCD) + q;         // position in the die-major sequence
    const int panel = v / (PR * TN), within = v - panel * (PR * TN);
    const int rows = min(PR, TM - panel * PR);                            // (the last panel may be shorter)
    tile_n = within / rows; tile_m = panel * PR + within - tile_n * rows;
  }
  const int m0 = tile_m * BM;
  const int n0 = tile_n * (EPI == EPI_SWIGLU ? HALF : BN);
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
    pa[i] = a + (size_t)gm * K + kc * 8 + (size_t)blockIdx.z * ((K / GB_BK + gridDim.z - 1) / gridDim.z) * GB_BK;
  }
#pragma unroll
  for (int i = 0; i < DMA_W; ++i) {
    const int sl = i * THREADS + tid, row = sl >> 3, kc = (sl & 7) ^ (row & 7);
    pw[i] = w + (size_t)wrow(row) * K + kc * 8 + (size_t)blockIdx.z * ((K / GB_BK + gridDim.z - 1) / gridDim.z) * GB_BK;
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
  // gridDim.z > 1 (EPI_F32 only): workgroup z takes the z-th run of K slices and writes float slab z (consumers add the
  // slabs in order)
  const int ks_all = K / GB_BK, ks_per = (ks_all + (int)gridDim.z - 1) / (int)gridDim.z;
  const int ks_first = (int)blockIdx.z * ks_per;
  const int ks_total = ks_all - ks_first < ks_per ? ks_all - ks_first : ks_per;
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
    // ... and everyone's; every wave is done with slice ks - 1, whose stage is refilled next.  With loads that must
    // stay in flight across it the bare barrier instruction: __syncthreads() would drain them (its fence waits for
    // every load in flight); the asm statements on both sides keep the LDS reads where they are
    if (STAGES == 2) __syncthreads(); else __builtin_amdgcn_s_barrier();
    if (ks + STAGES - 1 < ks_total) issue(ks + STAGES - 1);
    else asm volatile("" ::: "memory");
    const char* As = gb_lds + (ks % STAGES) * STAGE_BYTES;
    const char* Ws = As + A_BYTES;
    // Fragment reads run ahead of the matrix cores inside the slice: the (k32, row tile) steps are one sequence, the
    // activation fragment of step t + PF is requested before the MFMAs of step t, the weight fragments of the next
    // k32 at the start of the current one - a wave then waits for an LDS round trip only at the head of a slice
    constexpr int KS32 = GB_BK / 32, STEPS = KS32 * MI, PF = STEPS > 3 ? 3 : STEPS - 1;
    constexpr int FWS = (NT + MI - 1) / MI;             // weight fragments of the next k32 requested per step
    auto ld_fw = [&](int k32, int j) -> uint4 {
      // EPI_SWIGLU: the first half of the tiles = this wave's gate columns, the second half = the matching up columns
      const int r = EPI == EPI_SWIGLU ? (j < NT / 2 ? wn * (NT * 8) + j * 16 : HALF + wn * (NT * 8) + (j - NT / 2) * 16)
                                      : wn * (NT * 16) + j * 16;
      return *reinterpret_cast<const uint4*>(Ws + (r + m16) * 128 + (sw0 ^ (k32 * 64)));   // chunk index ^ 4 per k32
    };
    auto ld_fa = [&](int t) -> uint4 {
      const int k32 = t / MI, i = t % MI;
      return *reinterpret_cast<const uint4*>(As + (wm * (MI * 16) + i * 16 + m16) * 128 + (sw0 ^ (k32 * 64)));
    };
    uint4 fw[2][NT], fa[PF + 1];
#pragma unroll
    for (int j = 0; j < NT; ++j) fw[0][j] = ld_fw(0, j);
#pragma unroll
    for (int t = 0; t < PF; ++t) fa[t] = ld_fa(t);
    __builtin_amdgcn_sched_group_barrier(0x100, NT + PF, 0);          // the slice's first fragments, all requested at once
#pragma unroll
    for (int t = 0; t < STEPS; ++t) {
      const int k32 = t / MI, i = t % MI;
      int reads = 0;
      if (k32 + 1 < KS32)
#pragma unroll
        for (int f = 0; f < FWS; ++f) if (i * FWS + f < NT) { fw[(k32 + 1) & 1][i * FWS + f] = ld_fw(k32 + 1, i * FWS + f); ++reads; }
      if (t + PF < STEPS) { fa[(t + PF) % (PF + 1)] = ld_fa(t + PF); ++reads; }
#pragma unroll
      for (int j = 0; j < NT; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fw[k32 & 1][j]),
                                                           __builtin_bit_cast(bf16x8, fa[t % (PF + 1)]), acc[i][j], 0, 0, 0);
      // keep this order in the instruction stream: the step's LDS reads, then its MFMAs (the scheduler otherwise
      // sinks every read to just before its first use, and the wave waits out each round trip)
      if (reads == 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      else if (reads == 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      else if (reads == 3) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, NT, 0);
    }
  }
  // acc[i][j][e]: row m0 + wm*MI*16 + i*16 + m16, column (tile j) + 4*g + e
  if constexpr (EPI == EPI_ROPE) {
    rope_epilogue<D, KT, MI, NT>(acc, ep, m0 + wm * (MI * 16), n0 + wn * (NT * 16), M, N, m16, g);
    return;
  }
  if constexpr (EPI == EPI_ROPE_DEC) {
    rope_epilogue_decode<D, KT, MI, NT>(acc, ep, m0 + wm * (MI * 16), n0 + wn * (NT * 16), M, N, m16, g);
    return;
  }
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
      float* o = (float*)out + (size_t)blockIdx.z * M * N + (size_t)gm * N;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int gn = n0 + wn * (NT * 16) + j * 16 + 4 * g;
        if (EPI == EPI_RESID) {                        // every element belongs to one lane of one workgroup: plain read-add-write
          if (gn + 3 < N && (N & 3) == 0) *reinterpret_cast<f32x4*>(o + gn) = *reinterpret_cast<const f32x4*>(o + gn) + acc[i][j];
          else for (int e = 0; e < 4; ++e) if (gn + e < N) o[gn + e] += acc[i][j][e];
        } else {
          if (gn + 3 < N && (N & 3) == 0) *reinterpret_cast<f32x4*>(o + gn) = acc[i][j];
          else for (int e = 0; e < 4; ++e) if (gn + e < N) o[gn + e] = acc[i][j][e];
        }
      }
    }
  }
}

template <int EPI, int BM, int BN, int WM, int WN, int STAGES = 2, int D = 128, typename KT = bf16_t>
void tile_launch(hipStream_t s, const bf16_t* a, const bf16_t* w, void* out, int M, int N, int K, const RopeEpi& ep = RopeEpi{}) {
  constexpr int LDS_BYTES = STAGES * (BM + BN) * GB_BK * 2;     // stages x (A tile + W tile)
  // opt-in to more than 64 KB of dynamic LDS: once per template instance, thread-safe (initialisation of a local static)
  static const hipError_t attr_once = hipFuncSetAttribute((const void*)k_gemm_tile<EPI, BM, BN, WM, WN, STAGES, D, KT>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  (void)attr_once;
  const int ncols = EPI == EPI_SWIGLU ? BN / 2 : BN;             // output columns per tile
  dim3 grid((N + ncols - 1) / ncols, (M + BM - 1) / BM);
  hipLaunchKernelGGL((k_gemm_tile<EPI, BM, BN, WM, WN, STAGES, D, KT>), grid, dim3(WM * WN * 64), LDS_BYTES, s, a, w, out, M, N, K, ep);
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

void launch_gemm_big_resid(hipStream_t s, const bf16_t* a, const bf16_t* w, float* x, int M, int N, int K) {
  tile_launch<EPI_RESID, 256, 256, 2, 4>(s, a, w, (void*)x, M, N, K);
}

void launch_gemm_big_swiglu(hipStream_t s, const bf16_t* a, const bf16_t* wgu, bf16_t* act, int M, int F, int K) {
  tile_launch<EPI_SWIGLU, 256, 256, 2, 4>(s, a, wgu, (void*)act, M, F, K);
}

// QKV projection of a prefill chunk with S3 (rotary embedding, gate logit, cache appends) as its epilogue: for bf16
// models with heads of 64 or 128 whose chunk rows are whole sequences of n positions; not for the per-loop-cache modes.
bool gemm_rope_applies(int M, int N, int K, int D) {
  const long tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
  return M >= 512 && tiles >= 128 && (K % GB_BK) == 0 && (D == 64 || D == 128) && N % D == 0;
}

// QKV projection of a decode step with S3 as its epilogue: 64-row x 128-column tiles (a wave = 16 rows x 128 columns),
// whole K, four LDS stages; one launch instead of the streaming kernel's K-range slabs + k_rope_append.  Measured in
// the decode step at batch 64: 192 rows (L = 3) 6.59 -> 6.42 ms, 256 rows (L = 4) 6.84 -> 6.71 ms, 128 rows equal, so
// it is used from 129 rows on.
bool gemm_rope_rows_applies(int M, int N, int K, int D) {
  return M > 128 && (K % GB_BK) == 0 && (D == 64 || D == 128) && N % 128 == 0;
}
void launch_gemm_rope_rows(hipStream_t s, const bf16_t* a, const bf16_t* wqkv, int M, int N, int K, const float* gate_w,
                           const float* gate_b, bf16_t* q_out, float* z_out, const KvView& kv, const int32_t* pos, int L,
                           const Dims& dm, const double* inv_freq, int mode, bool kv8) {
  RopeEpi ep{gate_w, gate_b, inv_freq, q_out, z_out, kv, 0, 0, dm.Hq, dm.Hkv, mode, pos, L};
  if (dm.D == 128) {
    if (kv8) tile_launch<EPI_ROPE_DEC, 64, 128, 4, 1, 4, 128, fp8_t>(s, a, wqkv, nullptr, M, N, K, ep);
    else tile_launch<EPI_ROPE_DEC, 64, 128, 4, 1, 4, 128, bf16_t>(s, a, wqkv, nullptr, M, N, K, ep);
  } else {
    if (kv8) tile_launch<EPI_ROPE_DEC, 64, 128, 4, 1, 4, 64, fp8_t>(s, a, wqkv, nullptr, M, N, K, ep);
    else tile_launch<EPI_ROPE_DEC, 64, 128, 4, 1, 4, 64, bf16_t>(s, a, wqkv, nullptr, M, N, K, ep);
  }
}

void launch_gemm_big_rope(hipStream_t s, const bf16_t* a, const bf16_t* wqkv, int M, int N, int K, const float* gate_w,
                          const float* gate_b, bf16_t* q_out, float* z_out, const KvView& kv, int n, int loop, const Dims& dm,
                          const double* inv_freq, int mode, bool kv8) {
  const RopeEpi ep{gate_w, gate_b, inv_freq, q_out, z_out, kv, n, loop, dm.Hq, dm.Hkv, mode, nullptr, 1};
  if (dm.D == 128) {
    if (kv8) tile_launch<EPI_ROPE, 256, 256, 4, 2, 2, 128, fp8_t>(s, a, wqkv, nullptr, M, N, K, ep);
    else tile_launch<EPI_ROPE, 256, 256, 4, 2>(s, a, wqkv, nullptr, M, N, K, ep);
  } else {
    if (kv8) tile_launch<EPI_ROPE, 256, 256, 4, 2, 2, 64, fp8_t>(s, a, wqkv, nullptr, M, N, K, ep);
    else tile_launch<EPI_ROPE, 256, 256, 4, 2, 2, 64, bf16_t>(s, a, wqkv, nullptr, M, N, K, ep);
  }
}

// Decode step: act[M, F] = silu(a Wg^T) * (a Wu^T) for up to 256 rows in one launch: all rows of the step in one
// tile, whole K, 32 gate + 32 up columns per workgroup, SwiGLU in the epilogue - no split-K slabs and no separate
// activation kernel.  With three or four LDS stages (deeper rings: equal) and the fragment reads running ahead of the
// matrix cores this beats the streaming kernel + activation kernel at every row count (batch 64: L = 2 step 6.13 -> 5.95 ms, non-looped
// 5.39 -> 5.29; batch 1: 1.66 -> 1.56 ms per token); the tile height follows the rows (64 / 128 / 256).
bool gemm_swiglu_rows_applies(int M, int F, int K) {
  // (larger row counts - several 256-row tiles - until the 256 x 256 prefill tiles fill the chip: 257..1024 rows
  // measured 4-6 % of the step faster than the streaming kernel, which reads the weights once per 128-row block)
  return M >= 1 && (K % GB_BK) == 0 && (F + 31) / 32 >= 128;   // enough 32-column tiles to occupy the chip
}

// Decode-sized projections with the plain float epilogue: 64-column row tiles x S runs of K slices (one float slab per
// run; consumers add them in order), S chosen so that about 256 workgroups share the work
int gemm_rows_split_slabs(int M, int N, int K) {
  const int tiles = ((N + 63) / 64) * ((M + 255) / 256);
  int S = 256 / tiles; if (S < 1) S = 1;      // (128 and 512 workgroups measured slower)
  const int ks = K / GB_BK; if (S > ks / 8) S = ks / 8 > 0 ? ks / 8 : 1;      // at least 8 slices per run (4: equal at batch 64, slower at batch 1; 16: slower)
  return S;
}
void launch_gemm_rows_split(hipStream_t s, const bf16_t* a, const bf16_t* w, float* c, int M, int N, int K) {
  const int S = gemm_rows_split_slabs(M, N, K);
  constexpr int LDS256 = 3 * (256 + 64) * GB_BK * 2, LDS128 = 3 * (128 + 64) * GB_BK * 2, LDS64 = 4 * (64 + 64) * GB_BK * 2;
  RopeEpi ep{};
  if (M <= 64) {
    static const hipError_t a1 = hipFuncSetAttribute((const void*)k_gemm_tile<EPI_F32, 64, 64, 2, 2, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS64); (void)a1;
    hipLaunchKernelGGL((k_gemm_tile<EPI_F32, 64, 64, 2, 2, 4>), dim3((N + 63) / 64, 1, S), dim3(256), LDS64, s, a, w, (void*)c, M, N, K, ep);
  } else if (M <= 128) {
    static const hipError_t a2 = hipFuncSetAttribute((const void*)k_gemm_tile<EPI_F32, 128, 64, 2, 2, 3>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS128); (void)a2;
    hipLaunchKernelGGL((k_gemm_tile<EPI_F32, 128, 64, 2, 2, 3>), dim3((N + 63) / 64, 1, S), dim3(256), LDS128, s, a, w, (void*)c, M, N, K, ep);
  } else {
    static const hipError_t a3 = hipFuncSetAttribute((const void*)k_gemm_tile<EPI_F32, 256, 64, 4, 2, 3>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS256); (void)a3;
    hipLaunchKernelGGL((k_gemm_tile<EPI_F32, 256, 64, 4, 2, 3>), dim3((N + 63) / 64, (M + 255) / 256, S), dim3(512), LDS256, s, a, w, (void*)c, M, N, K, ep);
  }
}


void launch_gemm_swiglu_rows(hipStream_t s, const bf16_t* a, const bf16_t* wgu, bf16_t* act, int M, int F, int K) {
  // Wide feed-forward blocks (at least 200 tiles of 64 hidden columns), more than 64 rows: 64 gate + 64 up columns per
  // tile - half as many workgroups, each taking the step's rows once for twice the columns (F = 16384, batch 64:
  // L = 2 / 3 / 4 step -2 / -5 / -5 %; 64 rows and fewer: +1-2 %, so those keep the narrow tile)
  if (M > 64 && (F + 63) / 64 >= 200) {
    if (M <= 128) { tile_launch<EPI_SWIGLU, 128, 128, 2, 2, 3>(s, a, wgu, (void*)act, M, F, K); return; }
    tile_launch<EPI_SWIGLU, 256, 128, 4, 2, 3>(s, a, wgu, (void*)act, M, F, K);
    return;
  }
  if (M <= 64) { tile_launch<EPI_SWIGLU, 64, 64, 2, 2, 4>(s, a, wgu, (void*)act, M, F, K); return; }
  if (M <= 128) { tile_launch<EPI_SWIGLU, 128, 64, 2, 2, 3>(s, a, wgu, (void*)act, M, F, K); return; }
  tile_launch<EPI_SWIGLU, 256, 64, 4, 2, 3>(s, a, wgu, (void*)act, M, F, K);
}

}  // namespace plt
