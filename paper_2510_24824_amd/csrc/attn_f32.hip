// Attention for the PLT_F32 configuration (tiny models, launch-bound): one wave64 per
// (row, query head).  Lanes stride over keys, each lane keeps its own online-softmax state
// (m, l, acc[D]); the 64 states are merged with wavefront shuffles.  Serves decode rows and
// prefill rows alike through RowMap.  Computes, per row of loop stage l:
//   l == 0 (or plain): y = Attn(q, K_share[0..p], V_share[0..p])            [first loop]
//   l >= 1           : y = g * SWA(q, own K/V, w) + (1-g) * Attn(q, K_share, V_share)
//                      with g = sigmoid(z)                                   [Alg. 3 l.2-5, Eq. 2]
#include "plt_internal.h"

namespace plt {

__device__ inline float wsum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline float wmax(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// softmax attention of the query in qs[] over keys j0..j1-1 of one stream; result -> ys[D] (LDS)
template <int D>
__device__ void attend_range(const float* qs, const float* __restrict__ kbase,
                             const float* __restrict__ vbase, int j0, int j1, float scale, float* ys) {
  const int lane = threadIdx.x;
  float m = -INFINITY, lsum = 0.f;
  float acc[D];
#pragma unroll
  for (int i = 0; i < D; ++i) acc[i] = 0.f;
  for (int j = j0 + lane; j < j1; j += 64) {
    const float* kr = kbase + (size_t)j * D;
    float s = 0.f;
#pragma unroll 8
    for (int i = 0; i < D; ++i) s = fmaf(qs[i], kr[i], s);
    s *= scale;
    float mn = fmaxf(m, s);
    float alpha = expf(m - mn);      // m = -inf -> 0
    float pw = expf(s - mn);
    lsum = lsum * alpha + pw;
    const float* vb = vbase + (size_t)(j >> 5) * (D * 32) + (j & 31);
#pragma unroll
    for (int i = 0; i < D; ++i) acc[i] = acc[i] * alpha + pw * vb[i * 32];
    m = mn;
  }
  float M = wmax(m);
  float sc = (m == -INFINITY) ? 0.f : expf(m - M);
  float Lt = wsum(lsum * sc);
  float inv = Lt > 0.f ? 1.0f / Lt : 0.f;
#pragma unroll
  for (int i = 0; i < D; ++i) {
    float t = wsum(acc[i] * sc);
    if (lane == 0) ys[i] = t * inv;
  }
}

template <int D>
__global__ __launch_bounds__(64) void k_attn_f32(const float* __restrict__ q, const float* __restrict__ z,
                                                 float* __restrict__ y, KvView kv, RowMap rm, Dims dm,
                                                 int plain) {
  __shared__ float qs[D];
  __shared__ float yg[D];
  __shared__ float yl[D];
  const int h = blockIdx.x, r = blockIdx.y, lane = threadIdx.x;
  const int Hq = dm.Hq, Hkv = dm.Hkv, G = Hq / Hkv, kh = h / G;
  int b, p, l;
  row_decode(rm, r, b, p, l);
  const int bg = kv.b0 + b;
  for (int i = lane; i < D; i += 64) qs[i] = q[((size_t)r * Hq + h) * D + i];
  __syncthreads();
  // exact expf keeps the float path within 1e-5 of the float64 reference
  const float scale = 1.0f / sqrtf((float)D);
  {
    size_t stream = (size_t)bg * Hkv + kh;
    const size_t coff = plain == 3 ? (size_t)l * kv.cache_stride : 0;      // per-loop caches (own-KV ablation)
    attend_range<D>(qs, (const float*)kv.k_share + coff + stream * kv.n_pad * D,
                    (const float*)kv.v_share + coff + stream * (size_t)kv.n_pad * D, 0, p + 1, scale, yg);
  }
  const bool gated = !plain && l > 0;
  if (gated) {
    if (rm.prefill) {
      size_t stream = (size_t)b * Hkv + kh;
      int lo = p - kv.w + 1; if (lo < 0) lo = 0;
      attend_range<D>(qs, (const float*)kv.k_loc + stream * kv.n_pad_loc * D,
                      (const float*)kv.v_loc + stream * (size_t)kv.n_pad_loc * D, lo, p + 1, scale, yl);
    } else {
      size_t stream = ((size_t)bg * kv.n_rings + (l - 1)) * Hkv + kh;
      int nv = p + 1 < kv.w ? p + 1 : kv.w;
      attend_range<D>(qs, (const float*)kv.k_ring + stream * kv.w_pad * D,
                      (const float*)kv.v_ring + stream * (size_t)kv.w_pad * D, 0, nv, scale, yl);
    }
  }
  __syncthreads();
  float g = 0.f;
  if (gated) {
    size_t zi = rm.prefill ? (size_t)r * Hq + h : ((size_t)b * (dm.L - 1) + (l - 1)) * Hq + h;
    g = 1.0f / (1.0f + expf(-z[zi]));
  }
  for (int i = lane; i < D; i += 64) {
    float v = gated ? g * yl[i] + (1.0f - g) * yg[i] : yg[i];
    y[((size_t)r * Hq + h) * D + i] = v;
  }
}

void launch_attn_f32(hipStream_t s, const float* q, const float* z, float* y, KvView kv, RowMap rm,
                     int R, Dims dm, int plain) {
  dim3 grid(dm.Hq, R);
  if (dm.D == 64)
    hipLaunchKernelGGL(k_attn_f32<64>, grid, dim3(64), 0, s, q, z, y, kv, rm, dm, plain);
  else
    hipLaunchKernelGGL(k_attn_f32<128>, grid, dim3(64), 0, s, q, z, y, kv, rm, dm, plain);
}

}  // namespace plt
