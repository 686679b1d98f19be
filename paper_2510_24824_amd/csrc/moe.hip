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
//   k_moe_bucket  one workgroup: stable counting sort of the R*k (row, slot) pairs by expert
//                                                                                -> off [E+1], pair [R*k]
//   k_moe_gemm<GU>    workgroup = (expert, 64 hidden columns): gathers the expert's rows into LDS and
//                     streams the gate and up weight strips once from HBM; SwiGLU in the epilogue
//                                                                                -> act [R*k, F] by list position
//   k_moe_gemm<DOWN>  workgroup = (expert, 128 model columns): act rows x the expert's down matrix, scaled
//                     by p_e, scattered to y [slot][row][d]: k slabs that the residual kernel adds in slot
//                     order (deterministic, no atomics)
// Experts nobody selected cost no weight traffic (their workgroups leave at once).
#include "plt_internal.h"

namespace plt {

typedef __attribute__((ext_vector_type(4))) float f32x4;

// ---------------------------------------------------------------------------------------------- router
template <typename T>
__global__ __launch_bounds__(256) void k_moe_route(const T* __restrict__ a, const T* __restrict__ wr,
                                                   int32_t* __restrict__ sel_e, float* __restrict__ sel_p,
                                                   int d, int E, int k) {
  extern __shared__ float sm_route[];       // [d] the row as float, then [E] logits
  float* xr = sm_route;
  float* lg = sm_route + d;
  const int r = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  for (int i = tid; i < d; i += 256) xr[i] = ld<T>(a + (size_t)r * d + i);
  __syncthreads();
  for (int e = wv; e < E; e += 4) {
    const T* w = wr + (size_t)e * d;
    float acc = 0.f;
    if constexpr (sizeof(T) == 2) {
      if ((d & 7) == 0) {
        for (int i = lane * 8; i < d; i += 512) {
          const uint4 v = *reinterpret_cast<const uint4*>(w + i);
          const unsigned u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            acc += xr[i + 2 * j] * bf16_to_f32((bf16_t)(u[j] & 0xffffu));
            acc += xr[i + 2 * j + 1] * bf16_to_f32((bf16_t)(u[j] >> 16));
          }
        }
      } else {
        for (int i = lane; i < d; i += 64) acc += xr[i] * ld<T>(w + i);
      }
    } else {
      for (int i = lane; i < d; i += 64) acc += xr[i] * ld<T>(w + i);
    }
#pragma unroll
    for (int o = 32; o; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) lg[e] = acc;
  }
  __syncthreads();
  if (wv != 0) return;
  // softmax over all E (<= 256) logits and the k largest, one wave: lane holds logits lane + 64 j
  float v[4];
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < 4; ++j) { const int idx = lane + 64 * j; v[j] = idx < E ? lg[idx] : -INFINITY; mx = fmaxf(mx, v[j]); }
#pragma unroll
  for (int o = 32; o; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) if (lane + 64 * j < E) sum += expf(v[j] - mx);
#pragma unroll
  for (int o = 32; o; o >>= 1) sum += __shfl_xor(sum, o);
  for (int t = 0; t < k; ++t) {
    float bv = v[0]; int bi = lane;            // lane's best: ascending j, strict >, so its lowest index wins ties
#pragma unroll
    for (int j = 1; j < 4; ++j) if (v[j] > bv) { bv = v[j]; bi = lane + 64 * j; }
#pragma unroll
    for (int o = 32; o; o >>= 1) {
      const float ov = __shfl_xor(bv, o); const int oi = __shfl_xor(bi, o);
      if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if (lane == 0) { sel_e[(size_t)r * k + t] = bi; sel_p[(size_t)r * k + t] = expf(bv - mx) / sum; }
    if (lane == (bi & 63)) {
      const int j = bi >> 6;
      if (j == 0) v[0] = -INFINITY; else if (j == 1) v[1] = -INFINITY; else if (j == 2) v[2] = -INFINITY; else v[3] = -INFINITY;
    }
  }
}

// ---------------------------------------------------------------------------------------------- bucket
// Stable counting sort of the P = R*k pairs (index i = row*k + slot) by expert: pair[off[e] .. off[e+1])
// lists expert e's pairs in increasing i.  One workgroup of 16 waves; wave w owns a contiguous span of
// pairs.  Counting: the lanes of a 64-pair chunk that share an expert are found by ballot, so positions
// follow from population counts and the result does not depend on any execution order.
__device__ inline void lane_counter_add(int (&c)[4], int j, int n) {
  if (j == 0) c[0] += n; else if (j == 1) c[1] += n; else if (j == 2) c[2] += n; else c[3] += n;
}
__device__ inline int lane_counter_get(const int (&c)[4], int j) {
  return j == 0 ? c[0] : (j == 1 ? c[1] : (j == 2 ? c[2] : c[3]));
}
__global__ __launch_bounds__(1024) void k_moe_bucket(const int32_t* __restrict__ sel_e, int32_t* __restrict__ off,
                                                     int32_t* __restrict__ pair, int P, int E) {
  __shared__ int cnt[16][256];
  __shared__ int offs[257];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int per = (((P + 15) / 16) + 63) & ~63;
  const int beg = wv * per < P ? wv * per : P;
  const int end = beg + per < P ? beg + per : P;
  int c[4] = {0, 0, 0, 0};                       // lane holds the counters of experts lane + 64 j
  for (int i0 = beg; i0 < end; i0 += 64) {
    const int i = i0 + lane;
    const int e = i < end ? sel_e[i] : -1;
    unsigned long long todo = __ballot(i < end);
    while (todo) {
      const int el = __shfl(e, __ffsll((long long)todo) - 1);
      const unsigned long long m = __ballot(e == el);
      if (lane == (el & 63)) lane_counter_add(c, el >> 6, __popcll(m));
      todo &= ~m;
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) cnt[wv][lane + 64 * j] = c[j];
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int e = 0; e < E; ++e) {
      offs[e] = run;
      for (int w = 0; w < 16; ++w) run += cnt[w][e];
    }
    offs[E] = run;
  }
  __syncthreads();
  if (tid <= E) off[tid] = offs[tid];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = lane + 64 * j;
    int b = e < E ? offs[e] : 0;
    for (int w = 0; w < wv; ++w) b += cnt[w][e];
    c[j] = b;
  }
  for (int i0 = beg; i0 < end; i0 += 64) {
    const int i = i0 + lane;
    const int e = i < end ? sel_e[i] : -1;
    unsigned long long todo = __ballot(i < end);
    while (todo) {
      const int el = __shfl(e, __ffsll((long long)todo) - 1);
      const unsigned long long m = __ballot(e == el);
      const int base = __shfl(lane_counter_get(c, el >> 6), el & 63);
      if (e == el) pair[base + __popcll(m & ((1ull << lane) - 1ull))] = i;
      if (lane == (el & 63)) lane_counter_add(c, el >> 6, __popcll(m));
      todo &= ~m;
    }
  }
}

// ---------------------------------------------------------------------------------------------- grouped GEMM
// c[rows of expert e][N] = rows x w[e][N][K]^T on the matrix cores.  The expert's rows (MT*16 at a time)
// sit in LDS, one K range of KR at a time; each of the 4 waves streams two 16-row strips of the expert's
// weight matrix straight from HBM into registers in MFMA A-operand layout (16 bytes per lane), 256 k per
// step, the next step prefetched while the current one is multiplied.  GU: the two strips are the gate
// and the up rows of the same 16 hidden columns, SwiGLU in the epilogue.
template <int MT, int KR, bool GU>
__global__ __launch_bounds__(256) void k_moe_gemm(const bf16_t* __restrict__ a, const bf16_t* __restrict__ w,
                                                  const int32_t* __restrict__ off, const int32_t* __restrict__ pair,
                                                  const float* __restrict__ sel_p, bf16_t* __restrict__ act_out,
                                                  float* __restrict__ y_out, int R, int N, int K, int topk) {
  extern __shared__ __attribute__((aligned(16))) bf16_t As_moe[];   // [MT*16][KR + 8]
  bf16_t* As = As_moe;
  constexpr int LDK = KR + 8, KH = 8, STEPS = KR / (32 * KH);
  static_assert(STEPS >= 2 && STEPS % 2 == 0, "two register buffers alternate over an even number of steps");
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, m16 = lane & 15, g = lane >> 4;
  const int e = blockIdx.y;
  const int beg = off[e], n_e = off[e + 1] - beg;
  if (n_e <= 0) return;
  // the two weight strips of this wave: first output column and first weight row of each
  int col0[2];
  const bf16_t* wp[2];
  if (GU) {
    col0[0] = col0[1] = (blockIdx.x * 4 + wv) * 16;
    int n = col0[0] + m16; if (n >= N) n = N - 1;
    wp[0] = w + ((size_t)e * 2 * N + n) * K + g * 8;
    wp[1] = w + ((size_t)e * 2 * N + N + n) * K + g * 8;
  } else {
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      col0[sb] = ((blockIdx.x * 4 + wv) * 2 + sb) * 16;
      int n = col0[sb] + m16; if (n >= N) n = N - 1;
      wp[sb] = w + ((size_t)e * N + n) * K + g * 8;
    }
  }
  const int n_rng = (K + KR - 1) / KR;
  uint4 bufA[2][KH], bufB[2][KH];
  auto wload = [&](uint4 (&f)[2][KH], int t, int rng) {
    const int k0 = rng * KR;
    const int kr = (K - k0 < KR) ? K - k0 : KR;
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
#pragma unroll
      for (int kk = 0; kk < KH; ++kk) {
        int ko = (t * KH + kk) * 32; if (ko + g * 8 + 8 > kr) ko = 0;      // beyond K: an in-range chunk (meets zeros in LDS)
        f[sb][kk] = *reinterpret_cast<const uint4*>(wp[sb] + k0 + ko);
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
        const int src_row = GU ? pair[beg + li] / topk : beg + li;
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
      const int src_row = GU ? pair[beg + li] / topk : beg + li;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (kc < kr) v = *reinterpret_cast<const uint4*>(a + (size_t)src_row * K + k0 + kc);
      *reinterpret_cast<uint4*>(&As[row * LDK + kc]) = v;
    }
  };
  f32x4 acc[2][MT];
  auto mac = [&](const uint4 (&f)[2][KH], int t) {
#pragma unroll
    for (int kk = 0; kk < KH; ++kk) {
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const uint4 af = *reinterpret_cast<const uint4*>(&As[(i * 16 + m16) * LDK + (t * KH + kk) * 32 + g * 8]);
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
          acc[sb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, f[sb][kk]),
                                                              __builtin_bit_cast(bf16x8, af), acc[sb][i], 0, 0, 0);
      }
      if ((kk & 1) == 1) __builtin_amdgcn_sched_barrier(0);
    }
  };
  // the wait for a prefetched weight step must not be merged into the LDS slice's wait: order them
  wload(bufA, 0, 0);
  for (int m0 = 0; m0 < n_e; m0 += MT * 16) {
#pragma unroll
    for (int sb = 0; sb < 2; ++sb)
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
    // acc[sb][i][c] = C[list row m0 + i*16 + m16][col0[sb] + 4*g + c]
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int li = m0 + i * 16 + m16;
      if (li >= n_e) continue;
      if (GU) {
        const int col = col0[0] + 4 * g;
        if (col >= N) continue;
        bf16_t o[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) { const float gt = acc[0][i][c]; o[c] = f32_to_bf16(gt / (1.0f + expf(-gt)) * acc[1][i][c]); }
        uint2 pk; pk.x = (unsigned)o[0] | ((unsigned)o[1] << 16); pk.y = (unsigned)o[2] | ((unsigned)o[3] << 16);
        *reinterpret_cast<uint2*>(act_out + (size_t)(beg + li) * N + col) = pk;
      } else {
        const int pr = pair[beg + li];
        const int row = pr / topk, slot = pr - row * topk;
        const float p = sel_p[pr];
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) {
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
size_t moe_index_bytes(int R, int k, int E) {
  auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
  return 3 * al((size_t)R * k * 4) + al((size_t)(E + 1) * 4);
}
MoeIndex moe_index_carve(void* base, int R, int k, int E) {
  auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
  char* p = (char*)base;
  MoeIndex mi;
  mi.sel_e = (int32_t*)p; p += al((size_t)R * k * 4);
  mi.sel_p = (float*)p;   p += al((size_t)R * k * 4);
  mi.pair = (int32_t*)p;  p += al((size_t)R * k * 4);
  mi.off = (int32_t*)p;
  return mi;
}

template <int MT, int KR, bool GU>
static void moe_gemm_launch(hipStream_t s, dim3 grid, const bf16_t* a, const bf16_t* w, const MoeIndex& mi, bf16_t* act,
                            float* y, int R, int N, int K, int k) {
  const size_t lds = (size_t)MT * 16 * (KR + 8) * sizeof(bf16_t);
  static bool attr_done = false;     // one flag per template instance
  if (!attr_done) {
    (void)hipFuncSetAttribute((const void*)k_moe_gemm<MT, KR, GU>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_done = true;
  }
  hipLaunchKernelGGL((k_moe_gemm<MT, KR, GU>), grid, dim3(256), lds, s, a, w, mi.off, mi.pair, mi.sel_p, act, y, R, N, K, k);
}

// rows per LDS tile by the mean number of rows per expert: 32 (two workgroups per compute unit, K range
// 1024), 64 (two per unit, K range 512) or 128 (prefill-sized batches)
template <bool GU>
static void moe_gemm_pick(hipStream_t s, dim3 grid, const bf16_t* a, const bf16_t* w, const MoeIndex& mi, bf16_t* act,
                          float* y, int R, int N, int K, int k, int E) {
  const long mean = ((long)R * k + E - 1) / E;
  if (mean <= 24) moe_gemm_launch<2, 1024, GU>(s, grid, a, w, mi, act, y, R, N, K, k);
  else if (mean <= 48) moe_gemm_launch<4, 512, GU>(s, grid, a, w, mi, act, y, R, N, K, k);
  else moe_gemm_launch<8, 512, GU>(s, grid, a, w, mi, act, y, R, N, K, k);
}

template <typename T>
void launch_moe_ffn(hipStream_t s, const T* a, const T* router, const T* wgu, const T* wdown, T* act, float* y,
                    MoeIndex mi, int R, int d, int F, int E, int k) {
  const int P = R * k;
  hipLaunchKernelGGL(k_moe_route<T>, dim3(R), dim3(256), (size_t)(d + E) * sizeof(float), s, a, router, mi.sel_e, mi.sel_p,
                     d, E, k);
  hipLaunchKernelGGL(k_moe_bucket, dim3(1), dim3(1024), 0, s, mi.sel_e, mi.off, mi.pair, P, E);
  if constexpr (sizeof(T) == 2) {
    moe_gemm_pick<true>(s, dim3((F + 63) / 64, E), (const bf16_t*)a, (const bf16_t*)wgu, mi, (bf16_t*)act, nullptr, R, F, d, k, E);
    moe_gemm_pick<false>(s, dim3((d + 127) / 128, E), (const bf16_t*)act, (const bf16_t*)wdown, mi, nullptr, y, R, d, F, k, E);
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

}  // namespace plt
