// Mixture-of-experts feed-forward of block f [appendix, "MoE Models Recipe": SwiGLU experts, k of E per
// token].  Reading taken for the router (the paper builds on OLMoE): logits r = W_r b on the normed row
// b, p = softmax(r) over all E experts, the k experts with the largest logits are evaluated (equal
// logits: lowest index first) and their outputs are summed with weights p_e, not renormalised.
//
// While decoding, the L loop stages of a position go through this layer as one batch [Sec. 2.2.1]: an
// expert's weights are read once for all the rows of all loop stages that selected it.
//
// Four launches per layer:
//   k_moe_route   one workgroup per row: router logits, softmax, top-k          -> sel_e, sel_p [R, k]
//                 (512 rows and more: k_moe_route_mfma, the logits of 16 or 32 rows at a time on the matrix cores)
//   k_moe_bucket  one workgroup: stable counting sort of the R*k (row, slot) pairs by expert
//                                                                                -> off [E+1], pair [R*k]
//   k_moe_gemm<GU>    workgroup = (expert, 64 hidden columns): gathers the expert's rows into LDS and
//                     streams the gate and up weight strips once from HBM; SwiGLU in the epilogue
//                                                                                -> act [R*k, F] by list position
//   k_moe_gemm<DOWN>  workgroup = (expert, 128 model columns): act rows x the expert's down matrix, scaled
//                     by p_e, scattered to y [slot][row][d]: k slabs that the residual kernel adds in slot
//                     order (deterministic, no atomics)
// Experts nobody selected cost no weight traffic (their workgroups leave at once).  Batches of up to 1024 rows
// (decode steps) skip k_moe_bucket: the grouped GEMMs derive their expert's list from sel_e themselves.
// Prefill-sized batches (hundreds of rows per expert) sort over many workgroups (k_moe_span_*) and run both
// GEMMs as k_moe_gemm_tile (256 x 256 tiles, matrix-core-bound).
#include "plt_internal.h"
#include <type_traits>

namespace plt {

typedef __attribute__((ext_vector_type(4))) float f32x4;

// ---------------------------------------------------------------------------------------------- router
// One workgroup of 8 waves per row.  Wave v owns experts v, v + 8, ...; it takes them 8 at a time with the
// loads of all 8 weight rows issued together (the router matrix is small and cache-resident: what costs
// here is load latency, not bytes).
constexpr int ROUTE_WAVES = 8, ROUTE_EB = 8;
// TA: type of the row (model dtype, or fp8_t: e4m3 codes with block scales a_sc of a low-bit model); T: router matrix
template <typename TA, typename T>
__global__ __launch_bounds__(ROUTE_WAVES * 64) void k_moe_route(const TA* __restrict__ a, const uint8_t* __restrict__ a_sc,
                                                                const T* __restrict__ wr,
                                                                int32_t* __restrict__ sel_e, float* __restrict__ sel_p,
                                                                int d, int E, int k) {
  extern __shared__ float sm_route[];       // [d] the row as float, then [E] logits
  float* xr = sm_route;
  float* lg = sm_route + d;
  const int r = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  if constexpr (sizeof(TA) == 1) {
    const int nbp = mx_ascale_row_bytes(d);
    if ((d & 3) == 0) {                                     // four codes (of one block) per thread: one round trip
      for (int i = tid * 4; i < d; i += ROUTE_WAVES * 64 * 4) {
        const unsigned q = *reinterpret_cast<const unsigned*>(a + (size_t)r * d + i);
        const int ex = (int)a_sc[(size_t)r * nbp + mx_ascale_index(i >> 5)] - 127;
#pragma unroll
        for (int c = 0; c < 4; ++c) xr[i + c] = ldexpf(e4m3_to_f32((fp8_t)((q >> (8 * c)) & 0xffu)), ex);
      }
    } else {
      for (int i = tid; i < d; i += ROUTE_WAVES * 64)
        xr[i] = ldexpf(e4m3_to_f32(a[(size_t)r * d + i]), (int)a_sc[(size_t)r * nbp + mx_ascale_index(i >> 5)] - 127);
    }
  } else if (sizeof(TA) == 2 && (d & 7) == 0) {           // 16 bytes per thread: the whole row in one round trip
    for (int i = tid * 8; i < d; i += ROUTE_WAVES * 64 * 8) {
      const uint4 q = *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(a) + (size_t)r * d + i);
      const unsigned u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int c = 0; c < 4; ++c) { xr[i + 2 * c] = bf16_to_f32((bf16_t)(u[c] & 0xffffu)); xr[i + 2 * c + 1] = bf16_to_f32((bf16_t)(u[c] >> 16)); }
    }
  } else {
    for (int i = tid; i < d; i += ROUTE_WAVES * 64) xr[i] = ld<TA>(a + (size_t)r * d + i);
  }
  __syncthreads();
  for (int e0 = wv; e0 < E; e0 += ROUTE_WAVES * ROUTE_EB) {
    float acc[ROUTE_EB];
#pragma unroll
    for (int j = 0; j < ROUTE_EB; ++j) acc[j] = 0.f;
    if (sizeof(T) == 2 && (d & 7) == 0) {
      for (int i = lane * 8; i < d; i += 512) {
        uint4 v[ROUTE_EB];
#pragma unroll
        for (int j = 0; j < ROUTE_EB; ++j) {
          int e = e0 + j * ROUTE_WAVES; if (e >= E) e = E - 1;            // clamped: computed, never stored
          v[j] = *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(wr) + (size_t)e * d + i);
        }
        float x[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) x[c] = xr[i + c];
#pragma unroll
        for (int j = 0; j < ROUTE_EB; ++j) {
          const unsigned u[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            acc[j] += x[2 * c] * bf16_to_f32((bf16_t)(u[c] & 0xffffu));
            acc[j] += x[2 * c + 1] * bf16_to_f32((bf16_t)(u[c] >> 16));
          }
        }
      }
    } else {
      for (int i = lane; i < d; i += 64) {
        const float x = xr[i];
#pragma unroll
        for (int j = 0; j < ROUTE_EB; ++j) {
          int e = e0 + j * ROUTE_WAVES; if (e >= E) e = E - 1;
          acc[j] += x * ld<T>(wr + (size_t)e * d + i);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < ROUTE_EB; ++j) {
      const float s = wave_add_f32(acc[j]);
      const int e = e0 + j * ROUTE_WAVES;
      if (lane == 0 && e < E) lg[e] = s;
    }
  }
  __syncthreads();
  if (wv != 0) return;
  // softmax over all E (<= 256) logits and the k largest, one wave: lane holds logits lane + 64 j
  // (the exchanges between lanes are data-parallel-primitive moves and row / half-wave swaps on the vector ALU;
  // wavefront shuffles through the LDS crossbar made this tail as long as the logits before it)
  float v[4];
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < 4; ++j) { const int idx = lane + 64 * j; v[j] = idx < E ? lg[idx] : -INFINITY; mx = fmaxf(mx, v[j]); }
  mx = wave_max_f32(mx);
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) if (lane + 64 * j < E) sum += expf(v[j] - mx);
  sum = wave_add_f32(sum);
  const float inv = 1.0f / sum;
  for (int t = 0; t < k; ++t) {
    float lv = v[0]; int li = lane;            // lane's best: ascending j, strict >, so its lowest index wins ties
#pragma unroll
    for (int j = 1; j < 4; ++j) if (v[j] > lv) { lv = v[j]; li = lane + 64 * j; }
    const float bv = wave_max_f32(lv);                                    // the largest logit left,
    const int bi = wave_min_i32(lv == bv ? li : 0x7fffffff);              // then the lowest index that has it
    if (lane == 0) { sel_e[(size_t)r * k + t] = bi; sel_p[(size_t)r * k + t] = expf(bv - mx) * inv; }
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = (lane + 64 * j == bi) ? -INFINITY : v[j];     // taken: out of the running
  }
}

// ---------------------------------------------------------------------------------------------- router, matrix cores
// The same router for batches of 512 rows and more, 16-bit router matrices, row lengths that are a multiple of 128:
// the logits of RB x 16 rows x all experts as 16x16x32 bf16 tiles (rows = A operand, router rows = B operand), so
// the router matrix is read from the last-level cache once per RB x 16 rows instead of once per row.  The KS
// waves of a workgroup split the 128-wide chunks of the rows among them and add their partial tiles through LDS
// in wave order (deterministic).  In a tile the 16 lanes that share lane / 16 hold all the logits of a row, so
// softmax and top-k run on 4 rows side by side in a wave without another exchange through LDS.
// 16384 rows of 2048, 64 experts: 370 -> 33 us.
template <typename TA, int CB, int RB, int KS>
__global__ __launch_bounds__(KS * 64) void k_moe_route_mfma(const TA* __restrict__ a, const uint8_t* __restrict__ a_sc,
                                                            const bf16_t* __restrict__ wr, int32_t* __restrict__ sel_e,
                                                            float* __restrict__ sel_p, int R, int d, int E, int k) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_route[];
  float* red = reinterpret_cast<float*>(lds_route);              // [KS][RB][CB][4][64]
  const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), m16 = lane & 15, g = lane >> 4;
  const int row0 = blockIdx.x * (16 * RB);
  const int n_ch = d >> 7;
  f32x4 acc[RB][CB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) acc[rb][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
  size_t arow[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) { int r = row0 + rb * 16 + m16; if (r >= R) r = R - 1; arow[rb] = (size_t)r; }   // clamped: computed, never stored
  int boff[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) { int e = cb * 16 + m16; if (e >= E) e = E - 1; boff[cb] = e * d + g * 8; }
  const int nbp = mx_ascale_row_bytes(d);
  for (int c = wv; c < n_ch; c += KS) {
    bf16x8 af[RB][4];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      if constexpr (sizeof(TA) == 1) {       // e4m3 codes of 32-wide block 4 c + j, times the block's power of two: exact in bf16
        const TA* ap = a + arow[rb] * d + c * 128 + g * 8;
        const uint8_t* scp = a_sc + arow[rb] * nbp + mx_ascale_index(c * 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint2 u = *reinterpret_cast<const uint2*>(ap + j * 32);
          const float sc = ldexpf(1.0f, (int)scp[mx_ascale_index(j)] - 127);
          const bf16x2 r0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(u.x, sc, false);
          const bf16x2 r1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(u.x, sc, true);
          const bf16x2 r2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(u.y, sc, false);
          const bf16x2 r3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(u.y, sc, true);
          af[rb][j] = __builtin_shufflevector(__builtin_shufflevector(r0, r1, 0, 1, 2, 3), __builtin_shufflevector(r2, r3, 0, 1, 2, 3),
                                              0, 1, 2, 3, 4, 5, 6, 7);
        }
      } else {
        const TA* ap = a + arow[rb] * d + c * 128 + g * 8;
#pragma unroll
        for (int j = 0; j < 4; ++j) af[rb][j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(ap + j * 32));
      }
    }
#pragma unroll
    for (int cb0 = 0; cb0 < CB; cb0 += 4) {
      uint4 bv[4][4];
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) bv[q][j] = *reinterpret_cast<const uint4*>(wr + boff[cb0 + q] + c * 128 + j * 32);
      // every load of the step is issued before the first product waits for one (left alone, the compiler
      // alternates two loads and a product: a dozen dependent round trips per chunk instead of one)
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int rb = 0; rb < RB; ++rb)
            acc[rb][cb0 + q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[rb][j], __builtin_bit_cast(bf16x8, bv[q][j]), acc[rb][cb0 + q], 0, 0, 0);
    }
  }
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int x = 0; x < 4; ++x) red[(((wv * RB + rb) * CB + cb) * 4 + x) * 64 + lane] = acc[rb][cb][x];
  __syncthreads();
  // Lane group g of the tiles holds rows 4 g + x of a block, lane m16 of the group the logits of experts cb * 16 +
  // m16: one (row block, x) pair is four rows side by side in a wave, and the RB * 4 pairs are dealt out over
  // the waves.  The 16-lane exchanges are data-parallel-primitive moves (a few cycles each instead of a trip
  // through the LDS crossbar).
  for (int item = wv; item < RB * 4; item += KS) {
    const int rb = item >> 2, x = item & 3;
    const int r = row0 + rb * 16 + 4 * g + x;
    float v[CB];
    float mx = -INFINITY;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      float t = red[(((0 * RB + rb) * CB + cb) * 4 + x) * 64 + lane];
      for (int w = 1; w < KS; ++w) t += red[(((w * RB + rb) * CB + cb) * 4 + x) * 64 + lane];       // wave order: deterministic
      v[cb] = cb * 16 + m16 < E ? t : -INFINITY;
      mx = fmaxf(mx, v[cb]);
    }
    mx = fmaxf(mx, row16_xchg<0>(mx)); mx = fmaxf(mx, row16_xchg<1>(mx));
    mx = fmaxf(mx, row16_xchg<2>(mx)); mx = fmaxf(mx, row16_xchg<3>(mx));
    float sum = 0.f;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) if (cb * 16 + m16 < E) sum += expf(v[cb] - mx);
    sum += row16_xchg<0>(sum); sum += row16_xchg<1>(sum);
    sum += row16_xchg<2>(sum); sum += row16_xchg<3>(sum);
    const float inv = 1.0f / sum;
    const bool writer = m16 == 0 && r < R;
    int32_t* const se = sel_e + (size_t)r * k;
    float* const sp = sel_p + (size_t)r * k;
    for (int t = 0; t < k; ++t) {
      float lv = v[0]; int li = m16;             // ascending cb, strict >: the lane's lowest index wins ties
#pragma unroll
      for (int cb = 1; cb < CB; ++cb) if (v[cb] > lv) { lv = v[cb]; li = cb * 16 + m16; }
      float bv = fmaxf(lv, row16_xchg<0>(lv)); bv = fmaxf(bv, row16_xchg<1>(bv));      // the row's largest logit,
      bv = fmaxf(bv, row16_xchg<2>(bv)); bv = fmaxf(bv, row16_xchg<3>(bv));
      int bi = lv == bv ? li : 0x7fffffff;                                             // then the lowest index that has it
      bi = min(bi, row16_xchg<0>(bi)); bi = min(bi, row16_xchg<1>(bi));
      bi = min(bi, row16_xchg<2>(bi)); bi = min(bi, row16_xchg<3>(bi));
      if (writer) { se[t] = bi; sp[t] = expf(bv - mx) * inv; }
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) v[cb] = (cb * 16 + m16 == bi) ? -INFINITY : v[cb];      // taken: out of the running
    }
  }
}

template <typename TA, int CB, int RB, int KS>
static void moe_route_mfma_launch(hipStream_t s, const TA* a, const uint8_t* a_sc, const bf16_t* wr, const MoeIndex& mi,
                                  int R, int d, int E, int k) {
  const size_t lds = (size_t)KS * RB * CB * 64 * sizeof(f32x4);       // at most 64 KiB for the instances below
  hipLaunchKernelGGL((k_moe_route_mfma<TA, CB, RB, KS>), dim3((R + 16 * RB - 1) / (16 * RB)), dim3(KS * 64), lds, s, a, a_sc, wr,
                     mi.sel_e, mi.sel_p, R, d, E, k);
}

// rows as TA (bf16, or e4m3 codes with block scales), router in bf16
template <typename TA>
static void moe_route(hipStream_t s, const TA* a, const uint8_t* a_sc, const bf16_t* wr, const MoeIndex& mi, int R, int d, int E,
                      int k) {
  // (below about 500 rows one workgroup per row is as fast: both are bound by the launch and two cold round trips)
  if (R >= 512 && (d & 127) == 0 && E <= 256 && (long)E * d < (1L << 31)) {
    const bool big = R >= 2048;                  // prefill-sized: two row blocks per wave halve the router traffic
    if (E <= 64) {
      if (big) moe_route_mfma_launch<TA, 4, 2, 4>(s, a, a_sc, wr, mi, R, d, E, k);
      else moe_route_mfma_launch<TA, 4, 1, 16>(s, a, a_sc, wr, mi, R, d, E, k);     // 16 waves: one chunk each at 2048-wide rows
    } else if (E <= 128) moe_route_mfma_launch<TA, 8, 1, 4>(s, a, a_sc, wr, mi, R, d, E, k);
    else moe_route_mfma_launch<TA, 16, 1, 4>(s, a, a_sc, wr, mi, R, d, E, k);
    return;
  }
  hipLaunchKernelGGL((k_moe_route<TA, bf16_t>), dim3(R), dim3(ROUTE_WAVES * 64), (size_t)(d + E) * sizeof(float), s, a, a_sc, wr,
                     mi.sel_e, mi.sel_p, d, E, k);
}

// ---------------------------------------------------------------------------------------------- bucket
// Stable counting sort of the P = R*k pairs (index i = row*k + slot) by expert: pair[off[e] .. off[e+1])
// lists expert e's pairs in increasing i.  One workgroup of 16 waves; wave w owns a contiguous span of
// pairs and walks it 64 pairs at a time: the chunk sits in one register across the wave, entry t is
// broadcast with a lane read, and lane (e mod 64) keeps the running counter of expert e -- positions
// follow from counts alone, so the result does not depend on any execution order.  The walk is a chain
// of vector instructions per pair, so it is kept to a handful: EW = ceil(E / 64) counters per lane.
// first walk of a wave's span [beg, end): c[j] (lane l) += number of pairs of expert l + 64 j
template <int EW>
__device__ inline void moe_walk_count(const int32_t* __restrict__ sel_e, int beg, int end, int lane, int (&c)[EW]) {
  for (int i0 = beg; i0 < end; i0 += 64) {
    const int v = i0 + lane < end ? sel_e[i0 + lane] : -1;
    const int nt = end - i0 < 64 ? end - i0 : 64;
    for (int t = 0; t < nt; ++t) {
      const int el = __builtin_amdgcn_readlane(v, t);
      if (EW == 1) { c[0] += lane == el; }
      else {
#pragma unroll
        for (int j = 0; j < EW; ++j) c[j] += lane + 64 * j == el;
      }
    }
  }
}
// second walk: c[j] (lane l) holds the next list position of expert l + 64 j; every pair is stored at its position
template <int EW>
__device__ inline void moe_walk_scatter(const int32_t* __restrict__ sel_e, int beg, int end, int lane, int (&c)[EW],
                                        int32_t* __restrict__ pair) {
  for (int i0 = beg; i0 < end; i0 += 64) {
    const int v = i0 + lane < end ? sel_e[i0 + lane] : -1;
    const int nt = end - i0 < 64 ? end - i0 : 64;
    int mypos = 0;                               // lane t ends up with the list position of entry i0 + t
    for (int t = 0; t < nt; ++t) {
      const int el = __builtin_amdgcn_readlane(v, t);
      int pos;
      if (EW == 1) { pos = __builtin_amdgcn_readlane(c[0], el); c[0] += lane == el; }
      else {
        int cj = c[0];
#pragma unroll
        for (int j = 1; j < EW; ++j) cj = (el >> 6) == j ? c[j] : cj;
        pos = __builtin_amdgcn_readlane(cj, el & 63);
#pragma unroll
        for (int j = 0; j < EW; ++j) c[j] += lane + 64 * j == el;
      }
      if (lane == t) mypos = pos;
    }
    if (lane < nt) pair[mypos] = i0 + lane;      // one store per chunk, after the loop
  }
}
// exclusive prefix over the EW * 64 per-expert totals held by threads tid < EW * 64 (one per thread) -> offs[0 .. EW*64]
template <int EW>
__device__ inline void moe_expert_offsets(int tot, int tid, int* offs /* LDS [EW*64+1] */, int* wave_tot /* LDS [EW] */) {
  const int lane = tid & 63, wv = tid >> 6;
  int incl = 0;
  if (tid < EW * 64) {
    incl = tot;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) { const int up = __shfl_up(incl, o); if (lane >= o) incl += up; }
    if (lane == 63) wave_tot[wv] = incl;
  }
  __syncthreads();
  if (tid < EW * 64) {
    int base = 0;
    for (int w = 0; w < wv; ++w) base += wave_tot[w];
    offs[tid] = base + incl - tot;
    if (tid == EW * 64 - 1) offs[EW * 64] = base + incl;
  }
  __syncthreads();
}

template <int EW>
__global__ __launch_bounds__(1024) void k_moe_bucket(const int32_t* __restrict__ sel_e, int32_t* __restrict__ off,
                                                     int32_t* __restrict__ pair, int P, int E) {
  __shared__ int cnt[16][EW * 64];
  __shared__ int offs[EW * 64 + 1];
  __shared__ int wave_tot[EW];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int per = (((P + 15) / 16) + 63) & ~63;
  const int beg = wv * per < P ? wv * per : P;
  const int end = beg + per < P ? beg + per : P;
  int c[EW];                                     // lane holds the counters of experts lane + 64 j
#pragma unroll
  for (int j = 0; j < EW; ++j) c[j] = 0;
  moe_walk_count<EW>(sel_e, beg, end, lane, c);
#pragma unroll
  for (int j = 0; j < EW; ++j) cnt[wv][lane + 64 * j] = c[j];
  __syncthreads();
  int tot = 0;
  if (tid < EW * 64) {
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += cnt[w][tid];
  }
  moe_expert_offsets<EW>(tot, tid, offs, wave_tot);
  if (tid <= E) off[tid] = offs[tid];          // experts >= E have no pairs: offs[E] is the total
#pragma unroll
  for (int j = 0; j < EW; ++j) {
    const int e = lane + 64 * j;
    int b = offs[e];
    for (int w = 0; w < wv; ++w) b += cnt[w][e];
    c[j] = b;
  }
  moe_walk_scatter<EW>(sel_e, beg, end, lane, c, pair);
}

// The same sort for prefill-sized batches (tens of thousands of pairs, where one workgroup's walk takes 0.6 ms):
// spans of MOE_SPAN pairs, one per wave, over as many workgroups as it takes, in three launches -- count per span,
// positions per (span, expert) by one workgroup, scatter per span.  Positions still follow from counts alone:
// the lists are the ones k_moe_bucket produces.
constexpr int MOE_SPAN = 256;
template <int EW>
__global__ __launch_bounds__(1024) void k_moe_span_count(const int32_t* __restrict__ sel_e, int32_t* __restrict__ span_cnt, int P) {
  const int lane = threadIdx.x & 63, sp = blockIdx.x * 16 + (threadIdx.x >> 6);
  const int beg = sp * MOE_SPAN;
  if (beg >= P) return;
  const int end = beg + MOE_SPAN < P ? beg + MOE_SPAN : P;
  int c[EW];
#pragma unroll
  for (int j = 0; j < EW; ++j) c[j] = 0;
  moe_walk_count<EW>(sel_e, beg, end, lane, c);
#pragma unroll
  for (int j = 0; j < EW; ++j) span_cnt[(size_t)sp * (EW * 64) + lane + 64 * j] = c[j];
}
// span_cnt [n_spans][EW*64]: in, the counts; out, the first list position of (span, expert)
template <int EW>
__global__ __launch_bounds__(1024) void k_moe_span_offsets(int32_t* __restrict__ span_cnt, int32_t* __restrict__ off, int n_spans, int E) {
  __shared__ int cnt[16][EW * 64];
  __shared__ int offs[EW * 64 + 1];
  __shared__ int wave_tot[EW];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int per = (n_spans + 15) / 16;
  const int s0 = wv * per < n_spans ? wv * per : n_spans, s1 = s0 + per < n_spans ? s0 + per : n_spans;
  int c[EW];
#pragma unroll
  for (int j = 0; j < EW; ++j) c[j] = 0;
  for (int sp = s0; sp < s1; ++sp)
#pragma unroll
    for (int j = 0; j < EW; ++j) c[j] += span_cnt[(size_t)sp * (EW * 64) + lane + 64 * j];
#pragma unroll
  for (int j = 0; j < EW; ++j) cnt[wv][lane + 64 * j] = c[j];
  __syncthreads();
  int tot = 0;
  if (tid < EW * 64) {
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += cnt[w][tid];
  }
  moe_expert_offsets<EW>(tot, tid, offs, wave_tot);
  if (tid <= E) off[tid] = offs[tid];
#pragma unroll
  for (int j = 0; j < EW; ++j) {
    const int e = lane + 64 * j;
    int b = offs[e];
    for (int w = 0; w < wv; ++w) b += cnt[w][e];
    c[j] = b;
  }
  for (int sp = s0; sp < s1; ++sp)
#pragma unroll
    for (int j = 0; j < EW; ++j) {
      const size_t idx = (size_t)sp * (EW * 64) + lane + 64 * j;
      const int v = span_cnt[idx];
      span_cnt[idx] = c[j];
      c[j] += v;
    }
}
template <int EW>
__global__ __launch_bounds__(1024) void k_moe_span_scatter(const int32_t* __restrict__ sel_e, const int32_t* __restrict__ span_base,
                                                           int32_t* __restrict__ pair, int P) {
  const int lane = threadIdx.x & 63, sp = blockIdx.x * 16 + (threadIdx.x >> 6);
  const int beg = sp * MOE_SPAN;
  if (beg >= P) return;
  const int end = beg + MOE_SPAN < P ? beg + MOE_SPAN : P;
  int c[EW];
#pragma unroll
  for (int j = 0; j < EW; ++j) c[j] = span_base[(size_t)sp * (EW * 64) + lane + 64 * j];
  moe_walk_scatter<EW>(sel_e, beg, end, lane, c, pair);
}
// the sort, whichever way: up to MOE_SORT_ONE pairs by the single workgroup
constexpr int MOE_SORT_ONE = 4096;
template <int EW>
static void moe_sort_launch(hipStream_t s, const MoeIndex& mi, int P, int E) {
  if (P <= MOE_SORT_ONE) {
    hipLaunchKernelGGL(k_moe_bucket<EW>, dim3(1), dim3(1024), 0, s, mi.sel_e, mi.off, mi.pair, P, E);
    return;
  }
  const int n_spans = (P + MOE_SPAN - 1) / MOE_SPAN, wgs = (n_spans + 15) / 16;
  hipLaunchKernelGGL(k_moe_span_count<EW>, dim3(wgs), dim3(1024), 0, s, mi.sel_e, mi.span, P);
  hipLaunchKernelGGL(k_moe_span_offsets<EW>, dim3(1), dim3(1024), 0, s, mi.span, mi.off, n_spans, E);
  hipLaunchKernelGGL(k_moe_span_scatter<EW>, dim3(wgs), dim3(1024), 0, s, mi.sel_e, mi.span, mi.pair, P);
}
static void moe_sort(hipStream_t s, const MoeIndex& mi, int P, int E) {
  if (E <= 64) moe_sort_launch<1>(s, mi, P, E);
  else if (E <= 128) moe_sort_launch<2>(s, mi, P, E);
  else moe_sort_launch<4>(s, mi, P, E);
}

// ---------------------------------------------------------------------------------------------- expert lists
// Decode-sized batches skip the sort kernel: every workgroup of the grouped GEMMs scans the R*k selections
// itself (a few KB, cache-resident) and derives its expert's list -- the pairs i = row*k + slot with
// sel_e[i] == e in increasing i -- and the list's first position beg = number of pairs of experts below e.
// Same order and positions as the sort kernel produces, so both paths give identical results.
constexpr int MOE_FLY_ROWS = 1024;          // longest expert list (= rows) handled this way; R*k <= 65535 as well
__device__ inline void moe_expert_list(const int32_t* __restrict__ sel_e, int P, int e, uint16_t* list /* LDS [MOE_FLY_ROWS] */,
                                       int* cnt /* LDS [8] */, int& beg, int& n_e) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int base = 0, n = 0;
  for (int i0 = 0; i0 < P; i0 += 256) {
    const int i = i0 + tid;
    const int v = i < P ? sel_e[i] : 0x7fffffff;
    const unsigned long long mlt = __ballot(v < e), meq = __ballot(v == e);
    if (lane == 0) { cnt[wv] = __popcll(mlt); cnt[4 + wv] = __popcll(meq); }
    __syncthreads();
    int before = 0, all_eq = 0, all_lt = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) { const int c = cnt[4 + w]; if (w < wv) before += c; all_eq += c; all_lt += cnt[w]; }
    if (v == e) list[n + before + __popcll(meq & ((1ull << lane) - 1ull))] = (uint16_t)i;
    n += all_eq; base += all_lt;
    __syncthreads();
  }
  beg = base; n_e = n;
}

// ---------------------------------------------------------------------------------------------- grouped GEMM
// c[rows of expert e][N] = rows x W_e[N][K]^T on the matrix cores.  The expert's rows (MT*16 at a time)
// sit in LDS, one K range of KR at a time; each of the 4 waves streams NS 16-row strips of the expert's
// weight matrix straight from HBM into registers (MFMA A operand, 16 bytes per lane), KH 32-wide chunks
// per step, the next step prefetched while the current one is multiplied.  The expert matrices of bf16
// models are stored strip by strip in exactly that load order (moe_wtile_index): a wave load is one
// contiguous KiB and a strip one contiguous stream, read with the non-temporal hint (every weight byte
// is used once per step).  GU: strips come in pairs, the gate and the up rows of the same 16 hidden
// columns, SwiGLU in the epilogue.
template <int MT, int KR, bool GU, int NS, int KH>
__global__ __launch_bounds__(256) void k_moe_gemm(const bf16_t* __restrict__ a, const bf16_t* __restrict__ w,
                                                  const int32_t* __restrict__ off, const int32_t* __restrict__ pair,
                                                  const int32_t* __restrict__ sel_e,
                                                  const float* __restrict__ sel_p, bf16_t* __restrict__ act_out,
                                                  float* __restrict__ y_out, int R, int N, int K, int topk) {
  __shared__ uint16_t s_list[MOE_FLY_ROWS];
  __shared__ int s_cnt[8];
  extern __shared__ __attribute__((aligned(16))) bf16_t As_moe[];   // [MT*16][KR + 8]
  bf16_t* As = As_moe;
  constexpr int LDK = KR + 8, STEPS = KR / (32 * KH);
  static_assert(STEPS >= 2 && STEPS % 2 == 0, "two register buffers alternate over an even number of steps");
  static_assert(!GU || NS % 2 == 0, "gate and up strips come in pairs");
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, m16 = lane & 15, g = lane >> 4;
  const int e = blockIdx.y;
  const bool fly = pair == nullptr;              // no sorted lists: derive this expert's list from the selections
  int beg, n_e;
  if (fly) moe_expert_list(sel_e, R * topk, e, s_list, s_cnt, beg, n_e);
  else { beg = off[e]; n_e = off[e + 1] - beg; }
  if (n_e <= 0) return;
  auto pair_at = [&](int li) -> int { return fly ? (int)s_list[li] : pair[beg + li]; };
  // this wave's weight strips: first output column of each and where its stream starts
  constexpr int NC = GU ? NS / 2 : NS;           // 16-column groups of the output per wave
  int col0[NC];
  const bf16_t* wp[NS];
  const int n_strips = N >> 4;                   // N is a multiple of 16
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    int strip = (blockIdx.x * 4 + wv) * NC + c;
    col0[c] = strip * 16;
    if (strip >= n_strips) strip = n_strips - 1;         // beyond N: a valid strip, its results are not stored
    if (GU) {
      wp[2 * c] = w + ((size_t)e * 2 * N + (size_t)strip * 16) * K + lane * 8;
      wp[2 * c + 1] = w + ((size_t)e * 2 * N + N + (size_t)strip * 16) * K + lane * 8;
    } else {
      wp[c] = w + ((size_t)e * N + (size_t)strip * 16) * K + lane * 8;
    }
  }
  const int n_rng = (K + KR - 1) / KR;
  uint4 bufA[NS][KH], bufB[NS][KH];
  auto wload = [&](uint4 (&f)[NS][KH], int t, int rng) {
    const int k0 = rng * KR;
    const int kr = (K - k0 < KR) ? K - k0 : KR;
#pragma unroll
    for (int sb = 0; sb < NS; ++sb)
#pragma unroll
      for (int kk = 0; kk < KH; ++kk) {
        int ko = (t * KH + kk) * 32; if (ko + 32 > kr) ko = 0;       // beyond K: an in-range chunk (meets zeros in LDS)
        f[sb][kk] = ldg16_stream(wp[sb] + (size_t)((k0 + ko) >> 5) * 512);
      }
  };
  const unsigned lds_as = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)As;
  // rows m0 .. m0 + MT*16 - 1 of the expert's list (beyond n_e: the last row again, never stored), K range rng
  auto load_slice = [&](int m0, int rng) {
    const int k0 = rng * KR;
    const int kr = (K - k0 < KR) ? K - k0 : KR;
    if (kr == KR) {
      for (int row = wv; row < MT * 16; row += 4) {
        int li = m0 + row; if (li >= n_e) li = n_e - 1;
        const int src_row = GU ? pair_at(li) / topk : beg + li;
        const bf16_t* src = a + (size_t)src_row * K + k0 + lane * 8;
#pragma unroll
        for (int seg = 0; seg < KR / 512; ++seg) {
          const unsigned dst = __builtin_amdgcn_readfirstlane(lds_as + (unsigned)(row * LDK + seg * 512) * 2u);
          unsigned keep_m0;                                          // m0 is left as it was found
          asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                       : "=&s"(keep_m0) : "s"(dst), "v"(src + seg * 512) : "memory");
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      return;
    }
    for (int ch = tid; ch < MT * 16 * (KR / 8); ch += 256) {       // ragged range: zero-filled beyond K
      const int row = ch / (KR / 8), kc = (ch % (KR / 8)) * 8;
      int li = m0 + row; if (li >= n_e) li = n_e - 1;
      const int src_row = GU ? pair_at(li) / topk : beg + li;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (kc < kr) v = *reinterpret_cast<const uint4*>(a + (size_t)src_row * K + k0 + kc);
      *reinterpret_cast<uint4*>(&As[row * LDK + kc]) = v;
    }
  };
  f32x4 acc[NS][MT];
  auto mac = [&](const uint4 (&f)[NS][KH], int t) {
#pragma unroll
    for (int kk = 0; kk < KH; ++kk) {
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const uint4 af = *reinterpret_cast<const uint4*>(&As[(i * 16 + m16) * LDK + (t * KH + kk) * 32 + g * 8]);
#pragma unroll
        for (int sb = 0; sb < NS; ++sb)
          acc[sb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f[sb][kk]),
                                                              __builtin_bit_cast(bf16x8, af), acc[sb][i], 0, 0, 0);
      }
      if ((kk & 1) == 1) __builtin_amdgcn_sched_barrier(0);
    }
  };
  wload(bufA, 0, 0);
  for (int m0 = 0; m0 < n_e; m0 += MT * 16) {
#pragma unroll
    for (int sb = 0; sb < NS; ++sb)
#pragma unroll
      for (int i = 0; i < MT; ++i) acc[sb][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int rng = 0; rng < n_rng; ++rng) {
      __syncthreads();                       // every wave is done with the previous slice
      load_slice(m0, rng);
      __syncthreads();
#pragma unroll
      for (int t = 0; t < STEPS; ++t) {      // STEPS is even: step 0 of any range is in bufA
        if (t + 1 < STEPS) { if (t & 1) wload(bufA, t + 1, rng); else wload(bufB, t + 1, rng); }
        else if (rng + 1 < n_rng) wload(bufA, 0, rng + 1);
        else if (m0 + MT * 16 < n_e) wload(bufA, 0, 0);
        if (t & 1) mac(bufB, t); else mac(bufA, t);
      }
    }
    // acc[sb][i][c] = C[list row m0 + i*16 + m16][column of strip sb + 4*g + c]
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int li = m0 + i * 16 + m16;
      if (li >= n_e) continue;
      if (GU) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          const int col = col0[c] + 4 * g;
          if (col >= N) continue;
          bf16_t o[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            const float gt = acc[2 * c][i][x];
            o[x] = f32_to_bf16(gt / (1.0f + expf(-gt)) * acc[2 * c + 1][i][x]);
          }
          uint2 pk; pk.x = (unsigned)o[0] | ((unsigned)o[1] << 16); pk.y = (unsigned)o[2] | ((unsigned)o[3] << 16);
          *reinterpret_cast<uint2*>(act_out + (size_t)(beg + li) * N + col) = pk;
        }
      } else {
        const int pr = pair_at(li);
        const int row = pr / topk, slot = pr - row * topk;
        const float p = sel_p[pr];
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          const int col = col0[c] + 4 * g;
          if (col >= N) continue;
          f32x4 o = acc[c][i];
          o[0] *= p; o[1] *= p; o[2] *= p; o[3] *= p;
          *reinterpret_cast<f32x4*>(y_out + ((size_t)slot * R + row) * N + col) = o;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------- float models
// one workgroup per (list position, 16 columns); a wave computes its 4 columns one after the other
__global__ __launch_bounds__(256) void k_moe_gu_f32(const float* __restrict__ a, const float* __restrict__ w,
                                                    const int32_t* __restrict__ sel_e, const int32_t* __restrict__ pair,
                                                    float* __restrict__ act, int F, int K, int topk) {
  const int li = blockIdx.x, lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int pr = pair[li], row = pr / topk, e = sel_e[pr];
  const float* x = a + (size_t)row * K;
  for (int c = 0; c < 4; ++c) {
    const int col = (blockIdx.y * 4 + wv) * 4 + c;
    if (col >= F) return;
    const float* wg = w + ((size_t)e * 2 * F + col) * K;
    const float* wu = w + ((size_t)e * 2 * F + F + col) * K;
    float gt = 0.f, up = 0.f;
    for (int i = lane; i < K; i += 64) { gt += x[i] * wg[i]; up += x[i] * wu[i]; }
#pragma unroll
    for (int o = 32; o; o >>= 1) { gt += __shfl_xor(gt, o); up += __shfl_xor(up, o); }
    if (lane == 0) act[(size_t)li * F + col] = gt / (1.0f + expf(-gt)) * up;
  }
}
__global__ __launch_bounds__(256) void k_moe_down_f32(const float* __restrict__ act, const float* __restrict__ w,
                                                      const int32_t* __restrict__ sel_e, const int32_t* __restrict__ pair,
                                                      const float* __restrict__ sel_p, float* __restrict__ y, int R, int N,
                                                      int K, int topk) {
  const int li = blockIdx.x, lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int pr = pair[li], row = pr / topk, slot = pr - row * topk, e = sel_e[pr];
  const float p = sel_p[pr];
  const float* x = act + (size_t)li * K;
  for (int c = 0; c < 4; ++c) {
    const int col = (blockIdx.y * 4 + wv) * 4 + c;
    if (col >= N) return;
    const float* wd = w + ((size_t)e * N + col) * K;
    float s = 0.f;
    for (int i = lane; i < K; i += 64) s += x[i] * wd[i];
#pragma unroll
    for (int o = 32; o; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) y[((size_t)slot * R + row) * N + col] = p * s;
  }
}

// ---------------------------------------------------------------------------------------------- launch
// (span, expert) counters of the multi-workgroup sort: spans of 256 pairs x the expert count rounded up to 64
static size_t moe_span_ints(int R, int k, int E) {
  return (((size_t)R * k + 255) / 256) * (size_t)(((E + 63) / 64) * 64);
}
size_t moe_index_bytes(int R, int k, int E) {
  auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
  return 3 * al((size_t)R * k * 4) + al((size_t)(E + 1) * 4) + al(moe_span_ints(R, k, E) * 4);
}
MoeIndex moe_index_carve(void* base, int R, int k, int E) {
  auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
  char* p = (char*)base;
  MoeIndex mi;
  mi.sel_e = (int32_t*)p; p += al((size_t)R * k * 4);
  mi.sel_p = (float*)p;   p += al((size_t)R * k * 4);
  mi.pair = (int32_t*)p;  p += al((size_t)R * k * 4);
  mi.off = (int32_t*)p;   p += al((size_t)(E + 1) * 4);
  mi.span = (int32_t*)p;
  return mi;
}

template <int MT, int KR, bool GU, int NS, int KH>
static void moe_gemm_launch(hipStream_t s, const bf16_t* a, const bf16_t* w, const MoeIndex& mi, bf16_t* act,
                            float* y, int R, int N, int K, int k, int E) {
  const size_t lds = (size_t)MT * 16 * (KR + 8) * sizeof(bf16_t);
  // opt-in to more than 64 KB of dynamic LDS: once per template instance, thread-safe (initialisation of a local static)
  static const hipError_t attr_once = hipFuncSetAttribute((const void*)k_moe_gemm<MT, KR, GU, NS, KH>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  (void)attr_once;
  const int cols_per_wg = 4 * 16 * (GU ? NS / 2 : NS);
  hipLaunchKernelGGL((k_moe_gemm<MT, KR, GU, NS, KH>), dim3((N + cols_per_wg - 1) / cols_per_wg, E), dim3(256), lds, s, a, w,
                     mi.off, mi.pair, mi.sel_e, mi.sel_p, act, y, R, N, K, k);
}

// rows per LDS tile by the mean number of rows per expert: 32 (two workgroups per compute unit, K range
// 1024), 64 (two per unit, K range 512) or 128 (prefill-sized batches)
template <bool GU>
static void moe_gemm_pick(hipStream_t s, const bf16_t* a, const bf16_t* w, const MoeIndex& mi, bf16_t* act,
                          float* y, int R, int N, int K, int k, int E) {
  const long mean = ((long)R * k + E - 1) / E;
  if (mean <= 20) moe_gemm_launch<2, 1024, GU, 2, 8>(s, a, w, mi, act, y, R, N, K, k, E);
  else if (mean <= 48) moe_gemm_launch<4, 512, GU, 2, 8>(s, a, w, mi, act, y, R, N, K, k, E);
  else moe_gemm_launch<8, 512, GU, 2, 8>(s, a, w, mi, act, y, R, N, K, k, E);
}

// ---------------------------------------------------------------------------------------------- prefill-sized batches
// Grouped GEMM for hundreds of rows per expert (matrix-core-bound): the tile algebra of the dense prefill GEMM
// (workgroup tile 256 list rows x 256 weight rows, K in slices of 64 through two LDS stages filled HBM -> LDS
// directly, 8 waves of 128 x 64) on one expert's sorted list.  The activation rows of a tile are gathered
// through the list (GU) or lie contiguous by list position (DOWN); the weight tile is read out of the expert's
// strip-ordered matrix chunk by chunk.  GU: the tile holds 128 gate rows and the matching 128 up rows,
// SwiGLU in the epilogue.  grid (column tiles, row-tile slots): slot s belongs to the expert whose run of
// ceil(n_e / 256) row tiles contains s; P/256 + E slots always suffice, the surplus workgroups leave at once.
// Consecutive workgroups are the column tiles of one row tile: a compute die keeps meeting the same 1 MB
// column block of the expert's matrix while that expert's row tiles pass by.
template <bool GU>
__global__ __launch_bounds__(512) void k_moe_gemm_tile(const bf16_t* __restrict__ a, const bf16_t* __restrict__ w,
                                                       const int32_t* __restrict__ off, const int32_t* __restrict__ pair,
                                                       const float* __restrict__ sel_p, bf16_t* __restrict__ act_out,
                                                       float* __restrict__ y_out, int R, int N, int K, int topk, int E) {
  constexpr int BM = 256, BN = 256, BK = 64, THREADS = 512, WN = 4, MI = 8, NT = 4, HALF = 128;
  constexpr int A_BYTES = BM * BK * 2, W_BYTES = BN * BK * 2, STAGE_BYTES = A_BYTES + W_BYTES;
  extern __shared__ __attribute__((aligned(16))) char mt_lds[];
  __shared__ int s_where[3];                         // expert, first list position, rows of the expert
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, m16 = lane & 15, g = lane >> 4;
  const int wm = wv / WN, wn = wv % WN;
  if (wv == 0) {
    // which expert owns row-tile slot blockIdx.y: lanes scan 64 experts at a time
    const int slot = blockIdx.y;
    int base = 0, found = -1;
    for (int e0 = 0; e0 < E && found < 0; e0 += 64) {
      const int e = e0 + lane;
      const int n_e = e < E ? off[e + 1] - off[e] : 0;
      const int nt = (n_e + BM - 1) / BM;
      int incl = nt;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) { const int v = __shfl_up(incl, o, 64); if (lane >= o) incl += v; }
      const bool mine = slot >= base + incl - nt && slot < base + incl;
      const unsigned long long bal = __builtin_amdgcn_ballot_w64(mine);
      if (bal) {
        found = e0 + __builtin_ctzll(bal);
        if (mine) { s_where[0] = e; s_where[1] = off[e] + (slot - (base + incl - nt)) * BM; s_where[2] = off[e + 1]; }
      }
      base += __shfl(incl, 63, 64);
    }
    if (found < 0 && lane == 0) s_where[0] = -1;
  }
  __syncthreads();
  const int e = s_where[0];
  if (e < 0) return;
  const int p0 = s_where[1], p_end = s_where[2];     // list positions [p0, min(p0 + 256, p_end)) are this tile's rows
  const int NR = GU ? 2 * N : N;                     // rows of one expert's matrix
  const int n0 = blockIdx.x * (GU ? HALF : BN);
  const bf16_t* we = w + (size_t)e * NR * K;
  // weight row behind local tile row r (rows beyond the matrix: clamped, their outputs are never stored)
  auto wrow = [&](int r) -> int {
    int gr;
    if (GU) { const int c = n0 + (r & (HALF - 1)); gr = r < HALF ? c : N + c; if (c >= N) gr = NR - 1; }
    else gr = n0 + r;
    return gr < NR ? gr : NR - 1;
  };
  // this thread's chunks: slot s = i*THREADS + tid -> tile row s/8, chunk (s%8) ^ (row%8)  (as in the dense kernel)
  const bf16_t* pa[4]; const bf16_t* pw[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int sl = i * THREADS + tid, row = sl >> 3, kc = (sl & 7) ^ (row & 7);
    int pos = p0 + row; if (pos >= p_end) pos = p_end - 1;
    const size_t src_row = GU ? (size_t)(pair[pos] / topk) : (size_t)pos;
    pa[i] = a + src_row * K + kc * 8;
    pw[i] = we + moe_wtile_index(wrow(row), kc * 8, K);          // + 1024 elements per slice of 64
  }
  const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)mt_lds;
  auto dma16 = [](const bf16_t* src, unsigned lds_wave_base) {   // lane l: 16 bytes -> LDS[lds_wave_base + 16 l]
    unsigned keep_m0;                                            // m0 is left as it was found
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep_m0) : "s"(lds_wave_base), "v"(src) : "memory");
  };
  auto issue = [&](int ks) {
    const unsigned stage = lds0 + (unsigned)(ks & 1) * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      dma16(pa[i] + ks * BK, stage + __builtin_amdgcn_readfirstlane((unsigned)(i * THREADS + wv * 64) * 16));
#pragma unroll
    for (int i = 0; i < 4; ++i)
      dma16(pw[i] + (size_t)ks * 1024, stage + A_BYTES + __builtin_amdgcn_readfirstlane((unsigned)(i * THREADS + wv * 64) * 16));
  };
  const int ks_total = K / BK;
  f32x4 acc[MI][NT];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int sw0 = (g ^ (m16 & 7)) * 16;
  issue(0);
  // down projection: where this lane's 8 output rows go and their weights p_e, requested now and used after the
  // K loop (two dependent loads that the epilogue would otherwise wait for with the matrix cores idle)
  int out_pr[MI]; float out_p[MI];
  if (!GU) {
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      int pos = p0 + wm * 128 + i * 16 + m16; if (pos >= p_end) pos = p_end - 1;
      out_pr[i] = pair[pos];
    }
#pragma unroll
    for (int i = 0; i < MI; ++i) out_p[i] = sel_p[out_pr[i]];
  }
  for (int ks = 0; ks < ks_total; ++ks) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of slice ks has landed
    __syncthreads();                                   // ... and everyone's; slice ks - 1 is no longer read
    if (ks + 1 < ks_total) issue(ks + 1);
    const char* As = mt_lds + (ks & 1) * STAGE_BYTES;
    const char* Ws = As + A_BYTES;
#pragma unroll
    for (int k32 = 0; k32 < BK / 32; ++k32) {
      const int sw = sw0 ^ (k32 * 64);
      uint4 fw[NT];
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        // GU: tiles 0, 1 = this wave's 32 gate columns, tiles 2, 3 = the matching up columns
        const int r = GU ? (j < NT / 2 ? wn * 32 + j * 16 : HALF + wn * 32 + (j - NT / 2) * 16) : wn * 64 + j * 16;
        fw[j] = *reinterpret_cast<const uint4*>(Ws + (r + m16) * 128 + sw);
      }
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const uint4 fa = *reinterpret_cast<const uint4*>(As + (wm * 128 + i * 16 + m16) * 128 + sw);
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fw[j]),
                                                             __builtin_bit_cast(bf16x8, fa), acc[i][j], 0, 0, 0);
      }
    }
  }
  // acc[i][j][x]: list row p0 + wm*128 + i*16 + m16, column (tile j) + 4 g + x
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int pos = p0 + wm * 128 + i * 16 + m16;
    if (pos >= p_end) continue;
    if (GU) {
      bf16_t* o = act_out + (size_t)pos * N;
#pragma unroll
      for (int j = 0; j < NT / 2; ++j) {
        const int gn = n0 + wn * 32 + j * 16 + 4 * g;
        if (gn >= N) continue;                       // N is a multiple of 16: whole groups of 4 columns
        float v[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) { const float gt = acc[i][j][x]; v[x] = gt * __builtin_amdgcn_rcpf(1.0f + __expf(-gt)) * acc[i][j + NT / 2][x]; }   // (as the dense tile kernel: the result is rounded to bf16)
        const f32x4 vv = {v[0], v[1], v[2], v[3]};                 // hardware conversion (nearest even), two instructions
        *reinterpret_cast<bf16x4*>(o + gn) = __builtin_convertvector(vv, bf16x4);
      }
    } else {
      const int pr = out_pr[i];
      const int row = pr / topk, slot = pr - row * topk;
      const float p = out_p[i];
      float* o = y_out + ((size_t)slot * R + row) * N;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int gn = n0 + wn * 64 + j * 16 + 4 * g;
        if (gn >= N) continue;
        f32x4 v = acc[i][j];
        v[0] *= p; v[1] *= p; v[2] *= p; v[3] *= p;
        *reinterpret_cast<f32x4*>(o + gn) = v;
      }
    }
  }
}

// rows per expert from which the tiled kernel is used, and what it needs of the shapes
static bool moe_gemm_tile_applies(int R, int k, int E, int N, int K) {
  return (long)R * k >= (long)E * 192 && (K % 64) == 0 && (N % 16) == 0;
}
template <bool GU>
static void moe_gemm_tile_launch(hipStream_t s, const bf16_t* a, const bf16_t* w, const MoeIndex& mi, bf16_t* act, float* y,
                                 int R, int N, int K, int k, int E) {
  constexpr int LDS_BYTES = 2 * (256 + 256) * 64 * 2;
  // opt-in to more than 64 KB of dynamic LDS: once per template instance, thread-safe (initialisation of a local static)
  static const hipError_t attr_once = hipFuncSetAttribute((const void*)k_moe_gemm_tile<GU>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  (void)attr_once;
  const int ncols = GU ? 128 : 256;
  const long P = (long)R * k;
  dim3 grid((N + ncols - 1) / ncols, (unsigned)(P / 256 + E));
  hipLaunchKernelGGL(k_moe_gemm_tile<GU>, grid, dim3(512), LDS_BYTES, s, a, w, mi.off, mi.pair, mi.sel_p, act, y, R, N, K, k, E);
}

template <typename T>
void launch_moe_ffn(hipStream_t s, const T* a, const T* router, const T* wgu, const T* wdown, T* act, float* y,
                    MoeIndex mi, int R, int d, int F, int E, int k) {
  const int P = R * k;
  if constexpr (sizeof(T) == 2) moe_route<bf16_t>(s, a, nullptr, router, mi, R, d, E, k);
  else
    hipLaunchKernelGGL((k_moe_route<T, T>), dim3(R), dim3(ROUTE_WAVES * 64), (size_t)(d + E) * sizeof(float), s, a,
                       (const uint8_t*)nullptr, router, mi.sel_e, mi.sel_p, d, E, k);
  // decode-sized batches of bf16 models: the grouped GEMMs find their lists themselves (mi.pair = null)
  const bool fly = sizeof(T) == 2 && R <= MOE_FLY_ROWS && P <= 65535;
  if (fly) mi.pair = nullptr;
  else moe_sort(s, mi, P, E);
  if constexpr (sizeof(T) == 2) {
    if (!fly && moe_gemm_tile_applies(R, k, E, F, d) && moe_gemm_tile_applies(R, k, E, d, F)) {
      moe_gemm_tile_launch<true>(s, (const bf16_t*)a, (const bf16_t*)wgu, mi, (bf16_t*)act, nullptr, R, F, d, k, E);
      moe_gemm_tile_launch<false>(s, (const bf16_t*)act, (const bf16_t*)wdown, mi, nullptr, y, R, d, F, k, E);
    } else {
      moe_gemm_pick<true>(s, (const bf16_t*)a, (const bf16_t*)wgu, mi, (bf16_t*)act, nullptr, R, F, d, k, E);
      moe_gemm_pick<false>(s, (const bf16_t*)act, (const bf16_t*)wdown, mi, nullptr, y, R, d, F, k, E);
    }
  } else {
    hipLaunchKernelGGL(k_moe_gu_f32, dim3(P, (F + 15) / 16), dim3(256), 0, s, a, wgu, mi.sel_e, mi.pair, act, F, d, k);
    hipLaunchKernelGGL(k_moe_down_f32, dim3(P, (d + 15) / 16), dim3(256), 0, s, act, wdown, mi.sel_e, mi.pair, mi.sel_p,
                       y, R, d, F, k);
  }
}
template void launch_moe_ffn<float>(hipStream_t, const float*, const float*, const float*, const float*, float*, float*,
                                    MoeIndex, int, int, int, int, int);
template void launch_moe_ffn<bf16_t>(hipStream_t, const bf16_t*, const bf16_t*, const bf16_t*, const bf16_t*, bf16_t*,
                                     float*, MoeIndex, int, int, int, int, int);

// ---------------------------------------------------------------------------------------------- low-bit experts
// The grouped GEMM on MXFP4 expert weights and MXFP8 rows (block-scaled matrix cores, operand layouts as in
// gemm_mx.hip).  Workgroup = (expert, 128 output columns, GU: 128 hidden columns); a wave streams 4 strips
// (GU: the gate and up strips of 32 hidden columns, so that a wave owns whole 32-wide blocks of the hidden
// vector and can quantise them to e4m3 in its epilogue).
typedef __attribute__((ext_vector_type(8))) int i32x8;

template <int MT, bool GU>
__global__ __launch_bounds__(256, MT <= 4 ? 2 : 1) void k_moe_gemm_mx(const uint8_t* __restrict__ a, const uint8_t* __restrict__ a_sc,
                                                     const uint8_t* __restrict__ w, const uint8_t* __restrict__ w_sc,
                                                     const int32_t* __restrict__ off, const int32_t* __restrict__ pair,
                                                     const int32_t* __restrict__ sel_e,
                                                     const float* __restrict__ sel_p, uint8_t* __restrict__ act_out,
                                                     uint8_t* __restrict__ act_sc_out, float* __restrict__ y_out,
                                                     int R, int N, int K, int topk) {
  __shared__ uint16_t s_list[MOE_FLY_ROWS];
  __shared__ int s_cnt[8];
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_moe_mx[];   // [MT*16][MX_LDA] codes, then [MT*16][MX_SB] scales
  uint8_t* As = lds_moe_mx;
  uint8_t* Ss = lds_moe_mx + MT * 16 * MX_LDA;
  constexpr int NS = 4;
  // (the wave number in a scalar register: the strips' base addresses then are scalar too and a lane adds only
  // its 16 lane / 4 lane bytes at the load, which saves the vector registers the accumulators need)
  const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), m16 = lane & 15, g = lane >> 4;
  const int e = blockIdx.y;
  const bool fly = pair == nullptr;              // no sorted lists: derive this expert's list from the selections
  int beg, n_e;
  if (fly) moe_expert_list(sel_e, R * topk, e, s_list, s_cnt, beg, n_e);
  else { beg = off[e]; n_e = off[e + 1] - beg; }
  if (n_e <= 0) return;
  auto pair_at = [&](int li) -> int { return fly ? (int)s_list[li] : pair[beg + li]; };
  const int n_chunks = K >> 7, n_cgrp = (n_chunks + 3) >> 2, n_rng = (K + MX_KR - 1) / MX_KR;
  const int NR = GU ? 2 * N : N;                                 // rows of one expert's matrix
  const int out_strips = N >> 4;
  // the wave's four weight streams: strip (within the expert's matrix) and output column of each
  int col0[NS];
  const uint8_t* wp[NS];
  const uint8_t* sp[NS];
#pragma unroll
  for (int sb = 0; sb < NS; ++sb) {
    int strip = GU ? (blockIdx.x * 4 + wv) * 2 + (sb & 1) : (blockIdx.x * 4 + wv) * 4 + sb;
    col0[sb] = strip * 16;
    if (strip >= out_strips) strip = out_strips - 1;             // beyond N: a valid strip, results not stored
    const int strip_abs = (GU && sb >= 2) ? out_strips + strip : strip;      // up rows follow the gate rows
    wp[sb] = w + (size_t)e * ((size_t)NR * K / 2) + (size_t)strip_abs * n_chunks * 1024;
    sp[sb] = w_sc + (size_t)e * mx_wscale_bytes(NR, K) + (size_t)strip_abs * n_cgrp * 256;
  }
  struct WBuf { uint4 q[NS][4]; unsigned sc[NS]; };
  WBuf bufA, bufB;
  auto wload = [&](WBuf& f, int h, int rng) {      // half h of K range rng: 4 chunks of codes + their scale dword
    const int cg = rng * 2 + h;
    const int cgs = cg < n_cgrp ? cg : n_cgrp - 1;                // beyond K: any finite scale will do
#pragma unroll
    for (int sb = 0; sb < NS; ++sb) {
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        int ch = cg * 4 + kk; if (ch >= n_chunks) ch = 0;         // beyond K: an in-range chunk (meets zero codes)
        f.q[sb][kk] = ldg16_stream(wp[sb] + (size_t)ch * 1024 + lane * 16);
      }
      f.sc[sb] = *reinterpret_cast<const unsigned*>(sp[sb] + (size_t)cgs * 256 + lane * 4);
    }
  };
  const unsigned lds_as = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)As;
  const int asb = mx_ascale_row_bytes(K);
  auto load_slice = [&](int m0, int rng) {
    const int k0 = rng * MX_KR;
    const int kr = (K - k0 < MX_KR) ? K - k0 : MX_KR;
    if (kr == MX_KR) {
      for (int row = wv; row < MT * 16; row += 4) {
        int li = m0 + row; if (li >= n_e) li = n_e - 1;
        const int src_row = GU ? pair_at(li) / topk : beg + li;
        const uint8_t* src = a + (size_t)src_row * K + k0 + lane * 16;
        const unsigned dst = __builtin_amdgcn_readfirstlane(lds_as + (unsigned)row * MX_LDA);
        unsigned keep_m0;                                          // m0 is left as it was found
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                     : "=&s"(keep_m0) : "s"(dst), "v"(src) : "memory");
      }
    } else {
      for (int ch = tid; ch < MT * 16 * (MX_KR / 16); ch += 256) {  // ragged range: zero-filled beyond K
        const int row = ch / (MX_KR / 16), kc = (ch % (MX_KR / 16)) * 16;
        int li = m0 + row; if (li >= n_e) li = n_e - 1;
        const int src_row = GU ? pair_at(li) / topk : beg + li;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (kc < kr) v = *reinterpret_cast<const uint4*>(a + (size_t)src_row * K + k0 + kc);
        *reinterpret_cast<uint4*>(&As[row * MX_LDA + kc]) = v;
      }
    }
    for (int ch = tid; ch < MT * 16 * 2; ch += 256) {               // two 16-byte scale groups per row and range
      const int row = ch >> 1, h = ch & 1;
      int li = m0 + row; if (li >= n_e) li = n_e - 1;
      const int src_row = GU ? pair_at(li) / topk : beg + li;
      const int cg = rng * 2 + h;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (cg * 16 < asb) v = *reinterpret_cast<const uint4*>(a_sc + (size_t)src_row * asb + cg * 16);
      *reinterpret_cast<uint4*>(&Ss[row * MX_SB + h * 16]) = v;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  };
  f32x4 acc[NS][MT];
  struct BFrag { uint4 lo, hi; };
  auto bload = [&](int h, int idx) {
    const int kk = idx / MT, i = idx - kk * MT;
    const uint8_t* ap = &As[(i * 16 + m16) * MX_LDA + (h * 4 + kk) * 128 + g * 16];
    BFrag r; r.lo = *reinterpret_cast<const uint4*>(ap); r.hi = *reinterpret_cast<const uint4*>(ap + 64);
    return r;
  };
  auto mac = [&](const WBuf& f, int h) {
    unsigned bsc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) bsc[i] = *reinterpret_cast<const unsigned*>(&Ss[(i * 16 + m16) * MX_SB + h * 16 + g * 4]);
    BFrag cur = bload(h, 0);
#pragma unroll
    for (int idx = 0; idx < 4 * MT; ++idx) {
      const int kk = idx / MT, i = idx - kk * MT;
      BFrag nxt = cur;
      if (idx + 1 < 4 * MT) nxt = bload(h, idx + 1);
      const i32x8 bv = {(int)cur.lo.x, (int)cur.lo.y, (int)cur.lo.z, (int)cur.lo.w, (int)cur.hi.x, (int)cur.hi.y, (int)cur.hi.z, (int)cur.hi.w};
#pragma unroll
      for (int sb = 0; sb < NS; ++sb) {
        const i32x8 av = {(int)f.q[sb][kk].x, (int)f.q[sb][kk].y, (int)f.q[sb][kk].z, (int)f.q[sb][kk].w, 0, 0, 0, 0};
        if (kk == 0) acc[sb][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, acc[sb][i], 4, 0, 0, (int)f.sc[sb], 0, (int)bsc[i]);
        else if (kk == 1) acc[sb][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, acc[sb][i], 4, 0, 1, (int)f.sc[sb], 1, (int)bsc[i]);
        else if (kk == 2) acc[sb][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, acc[sb][i], 4, 0, 2, (int)f.sc[sb], 2, (int)bsc[i]);
        else acc[sb][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, acc[sb][i], 4, 0, 3, (int)f.sc[sb], 3, (int)bsc[i]);
      }
      cur = nxt;
      __builtin_amdgcn_sched_barrier(0);
    }
    // keeps the compiler from moving this half's MFMAs into later blocks (and their operands alive until then)
#pragma unroll
    for (int sb = 0; sb < NS; ++sb)
#pragma unroll
      for (int i = 0; i < MT; ++i) asm volatile("" : "+v"(acc[sb][i]));
  };
  wload(bufA, 0, 0);
  for (int m0 = 0; m0 < n_e; m0 += MT * 16) {
#pragma unroll
    for (int sb = 0; sb < NS; ++sb)
#pragma unroll
      for (int i = 0; i < MT; ++i) acc[sb][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int rng = 0; rng < n_rng; ++rng) {
      __syncthreads();                       // every wave is done with the previous slice
      load_slice(m0, rng);
      __syncthreads();
      wload(bufB, 1, rng);
      mac(bufA, 0);
      wload(bufA, 0, rng + 1 < n_rng ? rng + 1 : 0);     // next range, or range 0 again for the next row tile (unused at the end)
      mac(bufB, 1);
    }
    const int nbp = mx_ascale_row_bytes(N);
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int li = m0 + i * 16 + m16;
      if (GU) {
        // hidden values of row li: columns col0[j] + 4 g + x (j = 0, 1); the 32-wide block = both strips x the 4 lane groups
        float h[2][4];
        float amax = 0.f;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            const float gt = acc[j][i][x];
            h[j][x] = gt / (1.0f + expf(-gt)) * acc[2 + j][i][x];
            amax = fmaxf(amax, fabsf(h[j][x]));
          }
        amax = row4_max_f32(amax);
        const int ex = mx_block_exponent(amax, 8);
        if (li < n_e && col0[0] < N) {
#pragma unroll
          for (int j = 0; j < 2; ++j)
            *reinterpret_cast<unsigned*>(act_out + (size_t)(beg + li) * N + col0[j] + 4 * g) = mx_pack4_e4m3(h[j][0], h[j][1], h[j][2], h[j][3], ex);
          if (g == 0) act_sc_out[(size_t)(beg + li) * nbp + mx_ascale_index(col0[0] >> 5)] = (uint8_t)(ex + 127);
        }
      } else {
        if (li >= n_e) continue;
        const int pr = pair_at(li);
        const int row = pr / topk, slot = pr - row * topk;
        const float p = sel_p[pr];
#pragma unroll
        for (int sb = 0; sb < NS; ++sb) {
          const int col = col0[sb] + 4 * g;
          if (col >= N) continue;
          f32x4 o = acc[sb][i];
          o[0] *= p; o[1] *= p; o[2] *= p; o[3] *= p;
          *reinterpret_cast<f32x4*>(y_out + ((size_t)slot * R + row) * N + col) = o;
        }
      }
    }
  }
}

template <int MT, bool GU>
static void moe_gemm_mx_launch(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const uint8_t* w, const uint8_t* w_sc,
                               const MoeIndex& mi, uint8_t* act, uint8_t* act_sc, float* y, int R, int N, int K, int k, int E) {
  const size_t lds = (size_t)MT * 16 * (MX_LDA + MX_SB);
  // opt-in to more than 64 KB of dynamic LDS: once per template instance, thread-safe (initialisation of a local static)
  static const hipError_t attr_once = hipFuncSetAttribute((const void*)k_moe_gemm_mx<MT, GU>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  (void)attr_once;
  const int cols_per_wg = GU ? 128 : 256;
  hipLaunchKernelGGL((k_moe_gemm_mx<MT, GU>), dim3((N + cols_per_wg - 1) / cols_per_wg, E), dim3(256), lds, s, a, a_sc, w, w_sc,
                     mi.off, mi.pair, mi.sel_e, mi.sel_p, act, act_sc, y, R, N, K, k);
}

// Prefill-sized batches on low-bit operands: the grouping of k_moe_gemm_tile (row-tile slots over the experts' sorted
// lists, rows gathered through the list) around the tile algebra of the dense low-bit prefill kernel (256 list rows
// x 256 weight rows, one 128-wide chunk per LDS stage, weight strips as they lie in memory, scale dwords straight
// into registers).  GU: 8 gate strips and the matching 8 up strips per tile; a wave owns 32 hidden columns = one
// block, which it quantises to e4m3 in its epilogue.  DOWN: output scaled by p_e and scattered to the k slabs.
template <bool GU>
__global__ __launch_bounds__(512) void k_moe_gemm_mx_tile(const uint8_t* __restrict__ a, const uint8_t* __restrict__ a_sc,
                                                          const uint8_t* __restrict__ w, const uint8_t* __restrict__ w_sc,
                                                          const int32_t* __restrict__ off, const int32_t* __restrict__ pair,
                                                          const float* __restrict__ sel_p, uint8_t* __restrict__ act_out,
                                                          uint8_t* __restrict__ act_sc_out, float* __restrict__ y_out,
                                                          int R, int N, int K, int topk, int E) {
  constexpr int BM = 256, THREADS = 512, WN = 4, MI = 8, NT = 4;
  constexpr int A_BYTES = BM * 128, W_BYTES = 16 * 1024, STAGE_BYTES = A_BYTES + W_BYTES;
  extern __shared__ __attribute__((aligned(16))) char mxm_lds[];
  __shared__ int s_where[3];
  // (wave-uniform values in scalar registers, per-lane addresses as 32-bit offsets: the accumulators and operand
  // tuples leave few vector registers)
  const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), m16 = lane & 15, g = lane >> 4;
  const int wm = wv / WN, wn = wv % WN;
  if (wv == 0) {
    const int slot = blockIdx.y;
    int base = 0, found = -1;
    for (int e0 = 0; e0 < E && found < 0; e0 += 64) {
      const int e = e0 + lane;
      const int n_e = e < E ? off[e + 1] - off[e] : 0;
      const int nt = (n_e + BM - 1) / BM;
      int incl = nt;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) { const int v = __shfl_up(incl, o, 64); if (lane >= o) incl += v; }
      const bool mine = slot >= base + incl - nt && slot < base + incl;
      const unsigned long long bal = __builtin_amdgcn_ballot_w64(mine);
      if (bal) {
        found = e0 + __builtin_ctzll(bal);
        if (mine) { s_where[0] = e; s_where[1] = off[e] + (slot - (base + incl - nt)) * BM; s_where[2] = off[e + 1]; }
      }
      base += __shfl(incl, 63, 64);
    }
    if (found < 0 && lane == 0) s_where[0] = -1;
  }
  __syncthreads();
  const int e = __builtin_amdgcn_readfirstlane(s_where[0]);
  if (e < 0) return;
  const int p0 = __builtin_amdgcn_readfirstlane(s_where[1]), p_end = __builtin_amdgcn_readfirstlane(s_where[2]);
  const int NR = GU ? 2 * N : N, out_strips = N >> 4;
  const int n0 = blockIdx.x * (GU ? 128 : 256);
  const int n_chunks = K >> 7, n_cgrp = (n_chunks + 3) >> 2, asb = mx_ascale_row_bytes(K);
  const uint8_t* we = w + (size_t)e * ((size_t)NR * K / 2);
  const uint8_t* wse = w_sc + (size_t)e * mx_wscale_bytes(NR, K);
  // strip (within the expert's matrix) behind slot t of the tile's 16 weight strips
  auto strip_of = [&](int t) -> int {
    int st = (n0 >> 4) + (GU ? (t & 7) : t);
    if (st >= out_strips) st = out_strips - 1;                 // beyond N: a valid strip, results not stored
    return (GU && t >= 8) ? out_strips + st : st;
  };
  auto src_row = [&](int pos) -> size_t {
    if (pos >= p_end) pos = p_end - 1;
    return GU ? (size_t)(pair[pos] / topk) : (size_t)pos;
  };
  unsigned pa[4];                       // byte offsets into a (rows x K < 2^32)
  const uint8_t* pw[2];                 // per wave: scalar base, + 16 lane
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int sl = i * THREADS + tid, row = sl >> 3, pc = (sl & 7) ^ (row & 7);
    pa[i] = (unsigned)src_row(p0 + row) * (unsigned)K + pc * 16;
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) pw[i] = we + (size_t)strip_of(i * 8 + wv) * n_chunks * 1024;     // slot (i*512 + tid) / 64 = 8 i + wave
  const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)mxm_lds;
  auto dma16 = [](const uint8_t* src, unsigned lds_wave_base) {
    unsigned keep_m0;                                            // m0 is left as it was found
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep_m0) : "s"(lds_wave_base), "v"(src) : "memory");
  };
  auto issue = [&](int ch) {
    const unsigned stage = lds0 + (unsigned)(ch & 1) * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      dma16(a + ((size_t)pa[i] + (size_t)ch * 128), stage + (unsigned)(i * THREADS + wv * 64) * 16);
#pragma unroll
    for (int i = 0; i < 2; ++i)
      dma16(pw[i] + (size_t)ch * 1024 + lane * 16, stage + A_BYTES + (unsigned)(i * THREADS + wv * 64) * 16);
  };
  // the wave's four weight tiles: GU: slots 2 wn, 2 wn + 1 (gate) and 8 + 2 wn, 9 + 2 wn (up); DOWN: slots 4 wn ..
  int wslot[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) wslot[j] = GU ? (j < 2 ? wn * 2 + j : 8 + wn * 2 + (j - 2)) : wn * NT + j;
  const uint8_t* wsp[NT];               // per wave; + 4 lane
  unsigned asp[MI];                     // byte offsets into a_sc
#pragma unroll
  for (int j = 0; j < NT; ++j) wsp[j] = wse + (size_t)strip_of(wslot[j]) * n_cgrp * 256;
#pragma unroll
  for (int i = 0; i < MI; ++i) asp[i] = (unsigned)src_row(p0 + wm * 128 + i * 16 + m16) * (unsigned)asb + g * 4;
  unsigned wsc[NT], asc[MI], wsc_n[NT], asc_n[MI];
  auto load_scales = [&](int q, unsigned (&ws)[NT], unsigned (&as)[MI]) {
#pragma unroll
    for (int j = 0; j < NT; ++j) ws[j] = *reinterpret_cast<const unsigned*>(wsp[j] + (size_t)q * 256 + lane * 4);
#pragma unroll
    for (int i = 0; i < MI; ++i) as[i] = *reinterpret_cast<const unsigned*>(a_sc + ((size_t)asp[i] + q * 16));
  };
  f32x4 acc[MI][NT];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int sw0 = (g ^ (m16 & 7)) * 16;
  auto step = [&](int ch, auto kk_tag) {
    constexpr int kk = decltype(kk_tag)::value;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (ch + 1 < n_chunks) issue(ch + 1);
    const char* As = mxm_lds + (ch & 1) * STAGE_BYTES;
    const char* Ws = As + A_BYTES;
    uint4 fw[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) fw[j] = *reinterpret_cast<const uint4*>(Ws + wslot[j] * 1024 + lane * 16);
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const char* ap = As + (wm * 128 + i * 16 + m16) * 128;
      const uint4 lo = *reinterpret_cast<const uint4*>(ap + sw0), hi = *reinterpret_cast<const uint4*>(ap + (sw0 ^ 64));
      const i32x8 bv = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const i32x8 av = {(int)fw[j].x, (int)fw[j].y, (int)fw[j].z, (int)fw[j].w, 0, 0, 0, 0};
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, acc[i][j], 4, 0, kk, (int)wsc[j], kk, (int)asc[i]);
      }
    }
  };
  load_scales(0, wsc, asc);
  issue(0);
  for (int q = 0; q < n_cgrp; ++q) {
    const int ch0 = q * 4;
    step(ch0, std::integral_constant<int, 0>{});
    if (q + 1 < n_cgrp) load_scales(q + 1, wsc_n, asc_n);
    if (ch0 + 1 < n_chunks) step(ch0 + 1, std::integral_constant<int, 1>{});
    if (ch0 + 2 < n_chunks) step(ch0 + 2, std::integral_constant<int, 2>{});
    if (ch0 + 3 < n_chunks) step(ch0 + 3, std::integral_constant<int, 3>{});
    if (q + 1 < n_cgrp) {
#pragma unroll
      for (int j = 0; j < NT; ++j) wsc[j] = wsc_n[j];
#pragma unroll
      for (int i = 0; i < MI; ++i) asc[i] = asc_n[i];
    }
  }
  const int nbp = mx_ascale_row_bytes(N);
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int pos = p0 + wm * 128 + i * 16 + m16;
    if (GU) {
      // hidden values of list row pos, columns n0 + 32 wn + 16 j + 4 g + x (j = 0, 1): one 32-wide block over the 4 lane groups
      float h[2][4];
      float amax = 0.f;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          const float gt = acc[i][j][x];
          h[j][x] = gt * __builtin_amdgcn_rcpf(1.0f + __expf(-gt)) * acc[i][2 + j][x];   // (fast forms: the value is rounded to e4m3)
          amax = fmaxf(amax, fabsf(h[j][x]));
        }
      amax = row4_max_f32(amax);
      const int ex = mx_block_exponent(amax, 8);
      const int col = n0 + wn * 32;
      if (pos < p_end && col < N) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
          *reinterpret_cast<unsigned*>(act_out + (size_t)pos * N + col + j * 16 + 4 * g) = mx_pack4_e4m3(h[j][0], h[j][1], h[j][2], h[j][3], ex);
        if (g == 0) act_sc_out[(size_t)pos * nbp + mx_ascale_index(col >> 5)] = (uint8_t)(ex + 127);
      }
    } else {
      if (pos >= p_end) continue;
      const int pr = pair[pos];
      const int row = pr / topk, slot = pr - row * topk;
      const float p = sel_p[pr];
      float* o = y_out + ((size_t)slot * R + row) * N;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int gn = n0 + (wn * NT + j) * 16 + 4 * g;
        if (gn >= N) continue;
        f32x4 v = acc[i][j];
        v[0] *= p; v[1] *= p; v[2] *= p; v[3] *= p;
        *reinterpret_cast<f32x4*>(o + gn) = v;
      }
    }
  }
}
template <bool GU>
static void moe_gemm_mx_tile_launch(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const uint8_t* w, const uint8_t* w_sc,
                                    const MoeIndex& mi, uint8_t* act, uint8_t* act_sc, float* y, int R, int N, int K, int k, int E) {
  constexpr int LDS_BYTES = 2 * (256 * 128 + 16 * 1024);
  // opt-in to more than 64 KB of dynamic LDS: once per template instance, thread-safe (initialisation of a local static)
  static const hipError_t attr_once = hipFuncSetAttribute((const void*)k_moe_gemm_mx_tile<GU>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  (void)attr_once;
  const int ncols = GU ? 128 : 256;
  const long P = (long)R * k;
  dim3 grid((N + ncols - 1) / ncols, (unsigned)(P / 256 + E));
  hipLaunchKernelGGL(k_moe_gemm_mx_tile<GU>, grid, dim3(512), LDS_BYTES, s, a, a_sc, w, w_sc, mi.off, mi.pair, mi.sel_p, act, act_sc, y,
                     R, N, K, k, E);
}

void launch_moe_ffn_mx(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const bf16_t* router, const uint8_t* wgu,
                       const uint8_t* wgu_sc, const uint8_t* wdown, const uint8_t* wdown_sc, uint8_t* act_codes,
                       uint8_t* act_scales, float* y, MoeIndex mi, int R, int d, int F, int E, int k) {
  const int P = R * k;
  moe_route<fp8_t>(s, a, a_sc, router, mi, R, d, E, k);
  const bool fly = R <= MOE_FLY_ROWS && P <= 65535;
  if (fly) mi.pair = nullptr;
  else moe_sort(s, mi, P, E);
  const long mean = ((long)P + E - 1) / E;
  if (!fly && mean >= 192 && (d % 128) == 0 && (F % 128) == 0) {
    // prefill-sized: matrix-core-bound tiles (F % 128: whole 32-wide hidden blocks per wave, whole chunks for the down product)
    moe_gemm_mx_tile_launch<true>(s, a, a_sc, wgu, wgu_sc, mi, act_codes, act_scales, nullptr, R, F, d, k, E);
    moe_gemm_mx_tile_launch<false>(s, act_codes, act_scales, wdown, wdown_sc, mi, nullptr, nullptr, y, R, d, F, k, E);
  } else if (mean <= 20) {
    moe_gemm_mx_launch<2, true>(s, a, a_sc, wgu, wgu_sc, mi, act_codes, act_scales, nullptr, R, F, d, k, E);
    moe_gemm_mx_launch<2, false>(s, act_codes, act_scales, wdown, wdown_sc, mi, nullptr, nullptr, y, R, d, F, k, E);
  } else if (mean <= 48) {
    moe_gemm_mx_launch<4, true>(s, a, a_sc, wgu, wgu_sc, mi, act_codes, act_scales, nullptr, R, F, d, k, E);
    moe_gemm_mx_launch<4, false>(s, act_codes, act_scales, wdown, wdown_sc, mi, nullptr, nullptr, y, R, d, F, k, E);
  } else {
    moe_gemm_mx_launch<8, true>(s, a, a_sc, wgu, wgu_sc, mi, act_codes, act_scales, nullptr, R, F, d, k, E);
    moe_gemm_mx_launch<8, false>(s, act_codes, act_scales, wdown, wdown_sc, mi, nullptr, nullptr, y, R, d, F, k, E);
  }
}

}  // namespace plt
