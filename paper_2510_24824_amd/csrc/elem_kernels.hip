// Element-wise / row-wise kernels of the PLT step: micro-batch build, RMSNorm with residual
// accumulation, RoPE + gate logit + cache append, SwiGLU, carry update, argmax, layout packs.
// All are bandwidth-trivial next to attention and the projections; they are written for
// coalesced access and wave64 reductions, nothing more.
#include "plt_internal.h"

namespace plt {

__device__ inline float wave_sum(float v) {
  return wave_add_f32(v);
}

// block-wide sum for blockDim.x == 256 (4 waves)
__device__ inline float block_sum_256(float v, float* sm /*[4]*/) {
  v = wave_sum(v);
  int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm[w] = v;
  __syncthreads();
  return sm[0] + sm[1] + sm[2] + sm[3];
}

// ---- S0: displaced micro-batch [Alg. 1 l.5-6]; prefill: E + shift(H^(l-1)) [Alg. 2 l.4-5] ----
template <typename T>
__global__ void k_embed(const int32_t* __restrict__ tokens, const T* __restrict__ emb,
                        const float* __restrict__ carry, const float* __restrict__ hprev,
                        float* __restrict__ x, int d, RowMap rm, int n_loops, int add_prev, int vocab) {
  int r = blockIdx.x;
  int b, p, l;
  row_decode(rm, r, b, p, l);
  int tok = rm.prefill ? tokens[r] : tokens[b];
  tok = tok < 0 ? 0 : (tok >= vocab ? vocab - 1 : tok);   // ids outside the vocabulary are clamped
  const T* e = emb + (size_t)tok * d;
  const float* add = nullptr;
  if (add_prev && l > 0) {
    if (rm.prefill) { if (p > 0) add = hprev + (size_t)(r - 1) * d; }   // right shift by one
    else add = carry + ((size_t)b * (n_loops - 1) + (l - 1)) * d;        // H^l[p-1]
  }
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    float v = ld<T>(e + i);
    if (add) v += add[i];
    x[(size_t)r * d + i] = v;
  }
}
template <typename T>
void launch_embed(hipStream_t s, const int32_t* tokens, const T* emb, const float* carry,
                  const float* hprev, float* x, int R, int d, RowMap rm, int n_loops, int add_prev, int vocab) {
  hipLaunchKernelGGL(k_embed<T>, dim3(R), dim3(256), 0, s, tokens, emb, carry, hprev, x, d, rm,
                     n_loops, add_prev, vocab);
}
template void launch_embed<float>(hipStream_t, const int32_t*, const float*, const float*, const float*, float*, int, int, RowMap, int, int, int);
template void launch_embed<bf16_t>(hipStream_t, const int32_t*, const bf16_t*, const float*, const float*, float*, int, int, RowMap, int, int, int);

// ---- residual accumulation of GEMM slabs + RMSNorm (block f's two norms and the final norm) ----
template <typename T>
__global__ void k_resid_norm(float* __restrict__ x, int x_row_stride, int x_row_off,
                             const float* __restrict__ partials, int S, size_t slab,
                             const float* __restrict__ gain, float eps, T* __restrict__ a_out, int d) {
  __shared__ float sm[4];
  int r = blockIdx.x;
  float* xr = x + ((size_t)r * x_row_stride + x_row_off) * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += 256) {
    float v = xr[i];
    if (S > 0) {
      float acc = 0.f;
      for (int s = 0; s < S; ++s) acc += partials[(size_t)s * slab + (size_t)r * d + i];
      v += acc;
      xr[i] = v;
    }
    ss += v * v;
  }
  if (a_out == nullptr) return;
  ss = block_sum_256(ss, sm);
  float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int i = threadIdx.x; i < d; i += 256) st<T>(a_out + (size_t)r * d + i, xr[i] * inv * gain[i]);
}
// float4 variant for d % 4 == 0 and d <= 4096: every thread keeps its (up to 4) float4 values in
// registers between the accumulation and the normalisation pass, and the S slab loads of one
// value are issued together (independent accumulators) instead of one after the other.
template <typename T>
__global__ __launch_bounds__(256) void k_resid_norm4(float* __restrict__ x, int x_row_stride, int x_row_off,
                                                     const float* __restrict__ partials, int S, size_t slab,
                                                     const float* __restrict__ gain, float eps,
                                                     T* __restrict__ a_out, int d) {
  __shared__ float sm[4];
  const int r = blockIdx.x, d4 = d >> 2;
  float4* xr = reinterpret_cast<float4*>(x + ((size_t)r * x_row_stride + x_row_off) * d);
  float4 v[4];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int i = threadIdx.x + it * 256;
    if (i >= d4) break;
    float4 a = xr[i];
    if (S > 0) {
      const float4* pp = reinterpret_cast<const float4*>(partials + (size_t)r * d) + i;
      const size_t slab4 = slab >> 2;
      float4 acc0 = make_float4(0.f, 0.f, 0.f, 0.f), acc1 = acc0;
      int s = 0;
      for (; s + 4 <= S; s += 4) {
        float4 p0 = pp[(size_t)s * slab4], p1 = pp[(size_t)(s + 1) * slab4], p2 = pp[(size_t)(s + 2) * slab4],
               p3 = pp[(size_t)(s + 3) * slab4];
        acc0.x += p0.x; acc0.y += p0.y; acc0.z += p0.z; acc0.w += p0.w;
        acc1.x += p1.x; acc1.y += p1.y; acc1.z += p1.z; acc1.w += p1.w;
        acc0.x += p2.x; acc0.y += p2.y; acc0.z += p2.z; acc0.w += p2.w;
        acc1.x += p3.x; acc1.y += p3.y; acc1.z += p3.z; acc1.w += p3.w;
      }
      for (; s < S; ++s) {
        float4 p0 = pp[(size_t)s * slab4];
        acc0.x += p0.x; acc0.y += p0.y; acc0.z += p0.z; acc0.w += p0.w;
      }
      a.x += acc0.x + acc1.x; a.y += acc0.y + acc1.y; a.z += acc0.z + acc1.z; a.w += acc0.w + acc1.w;
      xr[i] = a;
    }
    v[it] = a;
    ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
  }
  if (a_out == nullptr) return;
  ss = block_sum_256(ss, sm);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int i = threadIdx.x + it * 256;
    if (i >= d4) break;
    const float4 gn = reinterpret_cast<const float4*>(gain)[i];
    T* dst = a_out + (size_t)r * d + 4 * i;
    st<T>(dst + 0, v[it].x * inv * gn.x); st<T>(dst + 1, v[it].y * inv * gn.y);
    st<T>(dst + 2, v[it].z * inv * gn.z); st<T>(dst + 3, v[it].w * inv * gn.w);
  }
}
template <typename T>
void launch_resid_norm(hipStream_t s, float* x, int x_row_stride, int x_row_off,
                       const float* partials, int S, size_t slab, const float* gain, float eps,
                       T* a_out, int R, int d) {
  if ((d & 3) == 0 && d <= 4096 && (slab & 3) == 0)
    hipLaunchKernelGGL(k_resid_norm4<T>, dim3(R), dim3(256), 0, s, x, x_row_stride, x_row_off, partials,
                       S, slab, gain, eps, a_out, d);
  else
    hipLaunchKernelGGL(k_resid_norm<T>, dim3(R), dim3(256), 0, s, x, x_row_stride, x_row_off, partials,
                       S, slab, gain, eps, a_out, d);
}
template void launch_resid_norm<float>(hipStream_t, float*, int, int, const float*, int, size_t, const float*, float, float*, int, int);
template void launch_resid_norm<bf16_t>(hipStream_t, float*, int, int, const float*, int, size_t, const float*, float, bf16_t*, int, int);

// Low-bit models: the same accumulation and RMSNorm, with the normed row quantised to e4m3 blocks of 32 on the
// way out (the input of the next low-bit projection).  A block is the 8 consecutive threads' float4 values.
__global__ __launch_bounds__(256) void k_resid_norm4_mx(float* __restrict__ x, const float* __restrict__ partials, int S,
                                                        size_t slab, const float* __restrict__ gain, float eps,
                                                        uint8_t* __restrict__ codes, uint8_t* __restrict__ scales, int d) {
  __shared__ float sm[4];
  const int r = blockIdx.x, d4 = d >> 2;
  float4* xr = reinterpret_cast<float4*>(x + (size_t)r * d);
  float4 v[4];
  float ss = 0.f;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int i = threadIdx.x + it * 256;
    if (i >= d4) break;
    float4 a = xr[i];
    if (S > 0) {
      const float4* pp = reinterpret_cast<const float4*>(partials + (size_t)r * d) + i;
      const size_t slab4 = slab >> 2;
      float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
      for (int s = 0; s < S; ++s) {
        const float4 p0 = pp[(size_t)s * slab4];
        acc.x += p0.x; acc.y += p0.y; acc.z += p0.z; acc.w += p0.w;
      }
      a.x += acc.x; a.y += acc.y; a.z += acc.z; a.w += acc.w;
      xr[i] = a;
    }
    v[it] = a;
    ss += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
  }
  ss = block_sum_256(ss, sm);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  const int nbp = mx_ascale_row_bytes(d);
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int i = threadIdx.x + it * 256;
    if (i >= d4) break;                 // d / 4 is a multiple of 8: a block's 8 threads leave together
    const float4 gn = reinterpret_cast<const float4*>(gain)[i];
    const float n0 = v[it].x * inv * gn.x, n1 = v[it].y * inv * gn.y, n2 = v[it].z * inv * gn.z, n3 = v[it].w * inv * gn.w;
    float amax = fmaxf(fmaxf(fabsf(n0), fabsf(n1)), fmaxf(fabsf(n2), fabsf(n3)));
    amax = fmaxf(amax, row16_xchg<0>(amax)); amax = fmaxf(amax, row16_xchg<1>(amax)); amax = fmaxf(amax, row16_xchg<2>(amax));   // 8 consecutive lanes
    const int e = mx_block_exponent(amax, 8);
    *reinterpret_cast<unsigned*>(codes + (size_t)r * d + 4 * i) = mx_pack4_e4m3(n0, n1, n2, n3, e);
    if ((i & 7) == 0) scales[(size_t)r * nbp + mx_ascale_index(i >> 3)] = (uint8_t)(e + 127);
  }
  if (threadIdx.x == 0) for (int b = d >> 5; b < nbp; ++b) scales[(size_t)r * nbp + mx_ascale_index(b)] = 0;
}
bool resid_norm_mx_applies(int d) { return (d & 31) == 0 && d <= 4096; }
void launch_resid_norm_mx(hipStream_t s, float* x, const float* partials, int S, size_t slab, const float* gain, float eps,
                          uint8_t* codes, uint8_t* scales, int R, int d) {
  hipLaunchKernelGGL(k_resid_norm4_mx, dim3(R), dim3(256), 0, s, x, partials, S, slab, gain, eps, codes, scales, d);
}

// SwiGLU over the gate/up slabs with the same quantiser on the way out: a thread owns 4 consecutive hidden
// columns of a row, 8 consecutive threads a block of 32
__global__ __launch_bounds__(256) void k_silu_mul_mx(const float* __restrict__ gu, int S, size_t slab, uint8_t* __restrict__ codes,
                                                     uint8_t* __restrict__ scales, int R, int F) {
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int f4 = F >> 2;
  const bool live = t < (size_t)R * f4;       // F / 4 is a multiple of 8: the 8 threads of a block are live together
  const int r = live ? (int)(t / f4) : 0, j = live ? (int)(t - (size_t)r * f4) : 0;
  float4 gt = make_float4(0.f, 0.f, 0.f, 0.f), up = gt;
  if (live)
    for (int s = 0; s < S; ++s) {
      const float* row = gu + (size_t)s * slab + (size_t)r * 2 * F;
      const float4 a = *reinterpret_cast<const float4*>(row + 4 * j), b = *reinterpret_cast<const float4*>(row + F + 4 * j);
      gt.x += a.x; gt.y += a.y; gt.z += a.z; gt.w += a.w; up.x += b.x; up.y += b.y; up.z += b.z; up.w += b.w;
    }
  const float h0 = gt.x / (1.0f + expf(-gt.x)) * up.x, h1 = gt.y / (1.0f + expf(-gt.y)) * up.y,
              h2 = gt.z / (1.0f + expf(-gt.z)) * up.z, h3 = gt.w / (1.0f + expf(-gt.w)) * up.w;
  float amax = fmaxf(fmaxf(fabsf(h0), fabsf(h1)), fmaxf(fabsf(h2), fabsf(h3)));
  amax = fmaxf(amax, row16_xchg<0>(amax)); amax = fmaxf(amax, row16_xchg<1>(amax)); amax = fmaxf(amax, row16_xchg<2>(amax));   // 8 consecutive lanes
  if (!live) return;
  const int e = mx_block_exponent(amax, 8), nbp = mx_ascale_row_bytes(F);
  *reinterpret_cast<unsigned*>(codes + (size_t)r * F + 4 * j) = mx_pack4_e4m3(h0, h1, h2, h3, e);
  if ((j & 7) == 0) scales[(size_t)r * nbp + mx_ascale_index(j >> 3)] = (uint8_t)(e + 127);
  if (j == 0) for (int b = F >> 5; b < nbp; ++b) scales[(size_t)r * nbp + mx_ascale_index(b)] = 0;
}
void launch_silu_mul_mx(hipStream_t s, const float* gu, int S, size_t slab, uint8_t* codes, uint8_t* scales, int R, int F) {
  const size_t n = (size_t)R * (F >> 2);
  hipLaunchKernelGGL(k_silu_mul_mx, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, gu, S, slab, codes, scales, R, F);
}

// ---- S3: RoPE, gate logit (Eq. 2, on the un-rotated query), cache append ----
// grid (ceil((Hq + 2*Hkv) / 4), R), 256 threads = 4 head vectors: lane j < D/2 of a wave owns the pair (j, j + D/2).
template <typename T, typename KT>
__global__ void k_rope_append(const float* __restrict__ qkv, int S, size_t slab,
                              const float* __restrict__ gate_w, const float* __restrict__ gate_b,
                              T* __restrict__ q_out, float* __restrict__ z_out, KvView kv, RowMap rm,
                              Dims dm, const double* __restrict__ inv_freq, int mode) {
  // mode: 0 = PLT (rings + gate), 1 = plain, 2 = loops >= 2 append nothing, 3 = row of loop l -> cache l
  // one wave per head vector, four head vectors per workgroup (fewer, fatter workgroups dispatch faster)
  const int hs = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6), r = blockIdx.y, j = threadIdx.x & 63;
  const int D = dm.D, half = D / 2, Hq = dm.Hq, Hkv = dm.Hkv;
  if (hs >= Hq + 2 * Hkv) return;
  const int ncol = (Hq + 2 * Hkv) * D;
  int b, p, l;
  row_decode(rm, r, b, p, l);
  const bool act = j < half;
  float lo = 0.f, hi = 0.f;
  if (act) {
    const float* src = qkv + (size_t)r * ncol + (size_t)hs * D;
    int s = 0;
    for (; s + 4 <= S; s += 4) {          // four slabs per round: eight independent loads in flight
      const float* p0 = src + (size_t)s * slab;
      float a0 = p0[j], b0 = p0[j + half], a1 = p0[slab + j], b1 = p0[slab + j + half];
      float a2 = p0[2 * slab + j], b2 = p0[2 * slab + j + half], a3 = p0[3 * slab + j], b3 = p0[3 * slab + j + half];
      lo += (a0 + a1) + (a2 + a3); hi += (b0 + b1) + (b2 + b3);
    }
    for (; s < S; ++s) { lo += src[(size_t)s * slab + j]; hi += src[(size_t)s * slab + j + half]; }
  }
  float c = 1.f, sn = 0.f;
  if (act && hs < Hq + Hkv) {
    // angle in turns, reduced in double (exact to ~1e-13), then a float sine / cosine
    double t = (double)p * inv_freq[j] * 0.15915494309189535;
    t -= rint(t);
    if (sizeof(T) == 2) {            // bf16 models: hardware sine / cosine of an angle given in turns
      sn = __builtin_amdgcn_sinf((float)t); c = __builtin_amdgcn_cosf((float)t);
    } else {
      sincosf((float)(t * 6.283185307179586), &sn, &c);
    }
  }
  if (hs < Hq) {
    if (mode == 0 && l > 0) {
      float zp = act ? lo * gate_w[hs * D + j] + hi * gate_w[hs * D + j + half] : 0.f;
      zp = wave_sum(zp);
      if (j == 0) {
        size_t zi = rm.prefill ? (size_t)r * Hq + hs
                               : ((size_t)b * (dm.L - 1) + (l - 1)) * Hq + hs;
        z_out[zi] = zp + gate_b[hs];
      }
    }
    if (act) {
      T* dst = q_out + (size_t)r * Hq * D + (size_t)hs * D;
      st<T>(dst + j, lo * c - hi * sn);
      st<T>(dst + j + half, hi * c + lo * sn);
    }
    return;
  }
  if (!act) return;
  const bool is_k = hs < Hq + Hkv;
  const int kh = is_k ? hs - Hq : hs - Hq - Hkv;
  float v0 = lo, v1 = hi;
  if (is_k) { v0 = lo * c - hi * sn; v1 = hi * c + lo * sn; }
  const int bg = kv.b0 + b;
  if (mode == 2 && l > 0) return;              // KV-share ablation: non-first loops keep no K/V
  if (mode != 0 || l == 0) {                   // first loop: the shared cache [Sec. 2.2.2]
    size_t stream = (size_t)bg * Hkv + kh;
    const size_t coff = mode == 3 ? (size_t)l * kv.cache_stride : 0;
    if (is_k) {
      KT* dst = (KT*)kv.k_share + coff + stream * (size_t)kv.n_pad * D;
      st<KT>(dst + kblk_index<KT>(p, j, D), v0); st<KT>(dst + kblk_index<KT>(p, j + half, D), v1);
    } else {
      KT* dst = (KT*)kv.v_share + coff + stream * (size_t)kv.n_pad * D;
      st<KT>(dst + vblk_index<KT>(p, j, D), v0); st<KT>(dst + vblk_index<KT>(p, j + half, D), v1);
    }
    return;
  }
  // non-first loop: only the w most recent entries survive (ring slot = p mod w)
  const int n = rm.rows_per_seq;
  if (rm.prefill) {
    size_t stream = (size_t)b * Hkv + kh;
    if (is_k) {
      KT* dst = (KT*)kv.k_loc + stream * (size_t)kv.n_pad_loc * D;
      st<KT>(dst + kblk_index<KT>(p, j, D), v0); st<KT>(dst + kblk_index<KT>(p, j + half, D), v1);
    } else {
      KT* dst = (KT*)kv.v_loc + stream * (size_t)kv.n_pad_loc * D;
      st<KT>(dst + vblk_index<KT>(p, j, D), v0); st<KT>(dst + vblk_index<KT>(p, j + half, D), v1);
    }
    if (p < n - kv.w) return;
  }
  {
    const int slot = p % kv.w;
    size_t stream = ((size_t)bg * kv.n_rings + (l - 1)) * Hkv + kh;
    if (is_k) {
      KT* dst = (KT*)kv.k_ring + stream * (size_t)kv.w_pad * D;
      st<KT>(dst + kblk_index<KT>(slot, j, D), v0); st<KT>(dst + kblk_index<KT>(slot, j + half, D), v1);
    } else {
      KT* dst = (KT*)kv.v_ring + stream * (size_t)kv.w_pad * D;
      st<KT>(dst + vblk_index<KT>(slot, j, D), v0); st<KT>(dst + vblk_index<KT>(slot, j + half, D), v1);
    }
  }
}
// ---- S3 for prefill-sized row counts: the same operation on tiles of 32 positions of one head ----
// N consecutive values -> N consecutive cache elements with one or two wide stores (dst suitably aligned)
template <int N>
__device__ inline void store_packed(bf16_t* dst, const float (&v)[N]) {
  unsigned w[N / 2];
#pragma unroll
  for (int i = 0; i < N / 2; ++i) w[i] = (unsigned)f32_to_bf16(v[2 * i]) | ((unsigned)f32_to_bf16(v[2 * i + 1]) << 16);
  if (N == 4) *reinterpret_cast<uint2*>(dst) = make_uint2(w[0], w[1]);
  else
#pragma unroll
    for (int i = 0; i < N / 8; ++i) reinterpret_cast<uint4*>(dst)[i] = make_uint4(w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]);
}
template <int N>
__device__ inline void store_packed(fp8_t* dst, const float (&v)[N]) {
  unsigned w[N / 4];
#pragma unroll
  for (int i = 0; i < N / 4; ++i) {
    float c[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) c[e] = fminf(fmaxf(v[4 * i + e], -448.f), 448.f);
    int pk = __builtin_amdgcn_cvt_pk_fp8_f32(c[0], c[1], 0, false);
    w[i] = (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(c[2], c[3], pk, true);
  }
  if (N == 4) *reinterpret_cast<unsigned*>(dst) = w[0];
  else if (N == 8) *reinterpret_cast<uint2*>(dst) = make_uint2(w[0], w[1]);
  else *reinterpret_cast<uint4*>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
}

// grid (ceil(n/32), Hq + 2*Hkv, Bc), 256 threads: thread (r = t/8, c = t%8) owns D/16 rotation pairs
// (j, j + D/2), j = c*D/16 .., of position p0 + r.  Q and K leave as 8- or 16-byte pieces (K straight into
// its tiled cache layout); V is transposed through LDS and leaves as the 16-byte chunks of one whole cache block.
template <int D, typename KT>
__global__ __launch_bounds__(256) void k_rope_append_tile(const float* __restrict__ qkv, int S, size_t slab,
                                                          const float* __restrict__ gate_w, const float* __restrict__ gate_b,
                                                          bf16_t* __restrict__ q_out, float* __restrict__ z_out, KvView kv,
                                                          int n, int loop, Dims dm, const double* __restrict__ inv_freq, int mode) {
  constexpr int PP = D / 16, half = D / 2;
  constexpr int PPT = 32 * D / 256;          // positions per thread when the V block is written out
  __shared__ float vt[D][33];
  const int t = threadIdx.x, r = t >> 3, jb = (t & 7) * PP;
  const int hs = blockIdx.y, b = blockIdx.z, p0 = blockIdx.x * 32, p = p0 + r;
  const int Hq = dm.Hq, Hkv = dm.Hkv, ncol = (Hq + 2 * Hkv) * D;
  const bool ok = p < n;
  const size_t row = (size_t)b * n + (ok ? p : 0);
  float lo[PP], hi[PP];
#pragma unroll
  for (int i = 0; i < PP; ++i) { lo[i] = 0.f; hi[i] = 0.f; }
  if (ok) {
    const float* src = qkv + row * ncol + (size_t)hs * D + jb;
    for (int s = 0; s < S; ++s) {
#pragma unroll
      for (int i = 0; i < PP / 4; ++i) {
        const float4 a = *reinterpret_cast<const float4*>(src + (size_t)s * slab + 4 * i);
        const float4 c = *reinterpret_cast<const float4*>(src + (size_t)s * slab + half + 4 * i);
        lo[4 * i] += a.x; lo[4 * i + 1] += a.y; lo[4 * i + 2] += a.z; lo[4 * i + 3] += a.w;
        hi[4 * i] += c.x; hi[4 * i + 1] += c.y; hi[4 * i + 2] += c.z; hi[4 * i + 3] += c.w;
      }
    }
  }
  const bool is_q = hs < Hq, is_k = !is_q && hs < Hq + Hkv;
  float rl[PP], rh[PP];
#pragma unroll
  for (int i = 0; i < PP; ++i) { rl[i] = lo[i]; rh[i] = hi[i]; }
  if (is_q || is_k) {
#pragma unroll
    for (int i = 0; i < PP; ++i) {
      // angle in turns, reduced in double, then the hardware sine / cosine (as in k_rope_append)
      double a = (double)p * inv_freq[jb + i] * 0.15915494309189535;
      a -= rint(a);
      const float sn = __builtin_amdgcn_sinf((float)a), c = __builtin_amdgcn_cosf((float)a);
      rl[i] = lo[i] * c - hi[i] * sn; rh[i] = hi[i] * c + lo[i] * sn;
    }
  }
  if (is_q) {
    if (mode == 0 && loop > 0) {                       // gate logit on the un-rotated query [Alg. 3 l.4]
      float zp = 0.f;
#pragma unroll
      for (int i = 0; i < PP; ++i) zp += lo[i] * gate_w[hs * D + jb + i] + hi[i] * gate_w[hs * D + half + jb + i];
      zp += row16_xchg<0>(zp); zp += row16_xchg<1>(zp); zp += row16_xchg<2>(zp);      // the 8 lanes of a position
      if (ok && (t & 7) == 0) z_out[row * Hq + hs] = zp + gate_b[hs];
    }
    if (ok) {
      bf16_t* dst = q_out + row * Hq * D + (size_t)hs * D + jb;
      store_packed<PP>(dst, rl); store_packed<PP>(dst + half, rh);
    }
    return;
  }
  if (mode == 2 && loop > 0) return;                   // KV-share ablation: non-first loops keep no K/V
  const int kh = is_k ? hs - Hq : hs - Hq - Hkv;
  const bool own = mode == 0 && loop > 0;              // non-first loop of the method: own K/V (+ ring tail)
  const size_t stream = own ? (size_t)b * Hkv + kh : (size_t)(kv.b0 + b) * Hkv + kh;
  const size_t stream_elems = (size_t)(own ? kv.n_pad_loc : kv.n_pad) * D;
  const bool ring = own && ok && p >= n - kv.w;        // the w most recent entries also enter the ring
  const int slot = p % kv.w;
  const size_t rstream = (((size_t)(kv.b0 + b) * kv.n_rings + (loop - 1)) * Hkv + kh) * (size_t)kv.w_pad * D;
  if (is_k) {
    if (ok) {
      KT* dst = (KT*)(own ? kv.k_loc : kv.k_share) + stream * stream_elems;
      store_packed<PP>(dst + kblk_index<KT>(p, jb, D), rl);
      store_packed<PP>(dst + kblk_index<KT>(p, jb + half, D), rh);
      if (ring) {
        KT* rd = (KT*)kv.k_ring + rstream;
        store_packed<PP>(rd + kblk_index<KT>(slot, jb, D), rl);
        store_packed<PP>(rd + kblk_index<KT>(slot, jb + half, D), rh);
      }
    }
    return;
  }
  // V: values are not rotated; transpose the tile through LDS and write the whole 32-position block
  if (ring) {
    KT* rd = (KT*)kv.v_ring + rstream;
#pragma unroll
    for (int i = 0; i < PP; ++i) { st<KT>(rd + vblk_index<KT>(slot, jb + i, D), lo[i]); st<KT>(rd + vblk_index<KT>(slot, jb + half + i, D), hi[i]); }
  }
#pragma unroll
  for (int i = 0; i < PP; ++i) { vt[jb + i][r] = lo[i]; vt[jb + half + i][r] = hi[i]; }   // zeros beyond the prompt
  __syncthreads();
  {
    const int d = t / (32 / PPT), q0 = (t % (32 / PPT)) * PPT;
    float o[PPT];
#pragma unroll
    for (int i = 0; i < PPT; ++i) o[i] = vt[d][q0 + i];
    // the thread's PPT consecutive positions of feature d: one or two 16-byte chunks of the blocked layout
    constexpr int CH = 16 / (int)sizeof(KT), RUN = PPT < CH ? PPT : CH;
    KT* dst = (KT*)(own ? kv.v_loc : kv.v_share) + stream * stream_elems;
#pragma unroll
    for (int c = 0; c < PPT / RUN; ++c) {
      float piece[RUN];
#pragma unroll
      for (int i = 0; i < RUN; ++i) piece[i] = o[c * RUN + i];
      store_packed<RUN>(dst + vblk_index<KT>(p0 + q0 + c * RUN, d, D), piece);
    }
  }
}

template <typename T, typename KT>
void launch_rope_append(hipStream_t s, const float* qkv, int S, size_t slab, const float* gate_w,
                        const float* gate_b, T* q_out, float* z_out, KvView kv, RowMap rm, int R,
                        Dims dm, const double* inv_freq, int mode) {
  if constexpr (sizeof(T) == 2) if (rm.prefill && mode != 3 && (slab & 3) == 0 && R % rm.rows_per_seq == 0 && rm.rows_per_seq >= 32) {
    // bf16 models, many positions per sequence: 32-position tiles with wide, contiguous cache stores
    const int n = rm.rows_per_seq, Bc = R / n;
    dim3 grid((n + 31) / 32, dm.Hq + 2 * dm.Hkv, Bc);
    if (dm.D == 128)
      hipLaunchKernelGGL((k_rope_append_tile<128, KT>), grid, dim3(256), 0, s, qkv, S, slab, gate_w, gate_b, (bf16_t*)q_out,
                         z_out, kv, n, rm.loop_fixed, dm, inv_freq, mode);
    else
      hipLaunchKernelGGL((k_rope_append_tile<64, KT>), grid, dim3(256), 0, s, qkv, S, slab, gate_w, gate_b, (bf16_t*)q_out,
                         z_out, kv, n, rm.loop_fixed, dm, inv_freq, mode);
    return;
  }
  hipLaunchKernelGGL((k_rope_append<T, KT>), dim3((dm.Hq + 2 * dm.Hkv + 3) / 4, R), dim3(256), 0, s, qkv, S, slab,
                     gate_w, gate_b, q_out, z_out, kv, rm, dm, inv_freq, mode);
}
template void launch_rope_append<float, float>(hipStream_t, const float*, int, size_t, const float*, const float*, float*, float*, KvView, RowMap, int, Dims, const double*, int);
template void launch_rope_append<bf16_t, bf16_t>(hipStream_t, const float*, int, size_t, const float*, const float*, bf16_t*, float*, KvView, RowMap, int, Dims, const double*, int);
template void launch_rope_append<bf16_t, fp8_t>(hipStream_t, const float*, int, size_t, const float*, const float*, bf16_t*, float*, KvView, RowMap, int, Dims, const double*, int);

// ---- SwiGLU: act = silu(gate) * up, gate = columns [0,F), up = columns [F,2F) ----
template <typename T>
__global__ void k_silu_mul(const float* __restrict__ gu, int S, size_t slab, T* __restrict__ act,
                           int R, int F) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)R * F) return;
  int r = (int)(i / F), f = (int)(i - (size_t)r * F);
  float g = 0.f, u = 0.f;
  for (int s = 0; s < S; ++s) {
    const float* row = gu + (size_t)s * slab + (size_t)r * 2 * F;
    g += row[f]; u += row[F + f];
  }
  st<T>(act + i, g / (1.0f + expf(-g)) * u);
}
template <typename T>
void launch_silu_mul(hipStream_t s, const float* gu, int S, size_t slab, T* act, int R, int F) {
  size_t n = (size_t)R * F;
  hipLaunchKernelGGL(k_silu_mul<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, gu, S, slab,
                     act, R, F);
}
template void launch_silu_mul<float>(hipStream_t, const float*, int, size_t, float*, int, int);
template void launch_silu_mul<bf16_t>(hipStream_t, const float*, int, size_t, bf16_t*, int, int);

// ---- greedy head: sum slabs, optional logits copy-out, argmax with lowest-index ties ----
// stage 1: grid (chunks, B): each block scans one chunk of the vocabulary; stage 2: one block per
// sequence merges the chunk winners.  Ties resolve to the lowest index in both stages.
constexpr int ARG_CHUNKS = 32;
__device__ inline void argmax_block_reduce(float best, int idx, float* bv, int* bi) {
  bv[threadIdx.x] = best; bi[threadIdx.x] = idx;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) {
      float v2 = bv[threadIdx.x + o]; int i2 = bi[threadIdx.x + o];
      if (v2 > bv[threadIdx.x] || (v2 == bv[threadIdx.x] && i2 < bi[threadIdx.x])) {
        bv[threadIdx.x] = v2; bi[threadIdx.x] = i2;
      }
    }
    __syncthreads();
  }
}
__global__ __launch_bounds__(256) void k_argmax_stage1(const float* __restrict__ lg, int S, size_t slab,
                                                       float* __restrict__ out, float* __restrict__ pv,
                                                       int* __restrict__ pi, int V) {
  __shared__ float bv[256];
  __shared__ int bi[256];
  const int b = blockIdx.y, ck = blockIdx.x;
  const int per = (V + ARG_CHUNKS - 1) / ARG_CHUNKS;
  const int i0 = ck * per, i1 = (i0 + per < V) ? i0 + per : V;
  float best = -INFINITY; int idx = 0x7fffffff;
  for (int i = i0 + threadIdx.x; i < i1; i += 256) {
    float v = 0.f;
    for (int s = 0; s < S; ++s) v += lg[(size_t)s * slab + (size_t)b * V + i];
    if (out) out[(size_t)b * V + i] = v;
    if (v > best) { best = v; idx = i; }
  }
  argmax_block_reduce(best, idx, bv, bi);
  if (threadIdx.x == 0) { pv[b * ARG_CHUNKS + ck] = bv[0]; pi[b * ARG_CHUNKS + ck] = bi[0]; }
}
__global__ void k_argmax_stage2(const float* __restrict__ pv, const int* __restrict__ pi,
                                int32_t* __restrict__ next) {
  const int b = blockIdx.x, t = threadIdx.x;             // 64 threads >= ARG_CHUNKS
  float v = t < ARG_CHUNKS ? pv[b * ARG_CHUNKS + t] : -INFINITY;
  int i = t < ARG_CHUNKS ? pi[b * ARG_CHUNKS + t] : 0x7fffffff;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    float v2 = __shfl_xor(v, o, 64); int i2 = __shfl_xor(i, o, 64);
    if (v2 > v || (v2 == v && i2 < i)) { v = v2; i = i2; }
  }
  if (t == 0) next[b] = i == 0x7fffffff ? 0 : i;
}
void launch_argmax(hipStream_t s, const float* lg, int S, size_t slab, float* logits_out, int32_t* next,
                   int B, int V, float* part_v, int* part_i) {
  hipLaunchKernelGGL(k_argmax_stage1, dim3(ARG_CHUNKS, B), dim3(256), 0, s, lg, S, slab, logits_out, part_v,
                     part_i, V);
  hipLaunchKernelGGL(k_argmax_stage2, dim3(B), dim3(64), 0, s, part_v, part_i, next);
}
int argmax_scratch_elems(int B) { return B * ARG_CHUNKS; }

// ---- S7: carried states for the next step: carry[b][l] = H^(l+1)[p], l = 0..L-2 ----
__global__ void k_carry_update(const float* __restrict__ x, float* __restrict__ carry, int L, int d) {
  int b = blockIdx.x / (L - 1), l = blockIdx.x % (L - 1);
  const float* src = x + ((size_t)b * L + l) * d;
  float* dst = carry + ((size_t)b * (L - 1) + l) * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) dst[i] = src[i];
}
void launch_carry_update(hipStream_t s, const float* x, float* carry, int B, int L, int d) {
  if (L <= 1) return;
  hipLaunchKernelGGL(k_carry_update, dim3(B * (L - 1)), dim3(256), 0, s, x, carry, L, d);
}
// prefill: carry[b0+b][l] = H^(l+1)[n-1] taken from the chunk's activation rows
__global__ void k_prefill_carry(const float* __restrict__ x, float* __restrict__ carry, int b0, int n,
                                int L, int l, int d) {
  int b = blockIdx.x;
  const float* src = x + ((size_t)b * n + (n - 1)) * d;
  float* dst = carry + ((size_t)(b0 + b) * (L - 1) + l) * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) dst[i] = src[i];
}
void launch_prefill_carry(hipStream_t s, const float* x, float* carry, int b0, int Bc, int n, int L,
                          int l, int d) {
  hipLaunchKernelGGL(k_prefill_carry, dim3(Bc), dim3(256), 0, s, x, carry, b0, n, L, l, d);
}

__global__ void k_pos_set(int32_t* pos, int B, int value, int increment) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < B) pos[i] = increment ? pos[i] + value : value;
}
void launch_pos_set(hipStream_t s, int32_t* pos, int B, int value, int increment) {
  hipLaunchKernelGGL(k_pos_set, dim3((B + 255) / 256), dim3(256), 0, s, pos, B, value, increment);
}

__global__ void k_copy_f32(const float* __restrict__ a, float* __restrict__ b, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) b[i] = a[i];
}
void launch_shift_copy(hipStream_t s, const float* x, float* hprev, size_t n) {
  unsigned g = (unsigned)((n + 255) / 256); if (g > 65536u) g = 65536u;
  hipLaunchKernelGGL(k_copy_f32, dim3(g), dim3(256), 0, s, x, hprev, n);
}

__global__ void k_fill_zero(uint4* __restrict__ p, size_t n16, unsigned char* __restrict__ tail, int n_tail) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  if (i < (size_t)n_tail) tail[i] = 0;
  for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}
void launch_fill_zero(hipStream_t s, void* p, size_t nbytes) {
  if (nbytes == 0) return;
  const size_t n16 = nbytes >> 4;
  size_t g = (n16 + 255) / 256; if (g < 1) g = 1; if (g > 8192) g = 8192;
  hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)g), dim3(256), 0, s, (uint4*)p, n16, (unsigned char*)p + (n16 << 4),
                     (int)(nbytes & 15));
}

// ---- layout packs: plain [S, n, D] <-> K [S, n_pad * D] (kblk_index order) / V [S, n_pad * D] (vblk_index order) ----
template <typename T>
__global__ void k_pack_k(const T* __restrict__ src, T* __restrict__ dst, int n, int n_pad, int D, int unpack) {
  int sidx = blockIdx.y;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;     // enumerates (pos, f) of the padded plain layout
  if (i >= (size_t)n_pad * D) return;
  int pos = (int)(i / D), f = (int)(i - (size_t)pos * D);
  const size_t li = (size_t)sidx * n_pad * D + kblk_index<T>(pos, f, D);
  if (unpack) {
    if (pos < n) dst[(size_t)sidx * n * D + i] = src[li];
  } else {
    T zero; st<T>(&zero, 0.f);
    dst[li] = pos < n ? src[(size_t)sidx * n * D + i] : zero;
  }
}
template <typename T>
__global__ void k_pack_v(const T* __restrict__ src, T* __restrict__ dst, int n, int n_pad, int D, int unpack) {
  int sidx = blockIdx.y;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;     // enumerates (pos, d) of the padded plain layout
  if (i >= (size_t)n_pad * D) return;
  int pos = (int)(i / D), dd = (int)(i - (size_t)pos * D);
  const size_t li = (size_t)sidx * n_pad * D + vblk_index<T>(pos, dd, D);
  if (unpack) {
    if (pos < n) dst[(size_t)sidx * n * D + i] = src[li];
  } else {
    T zero; st<T>(&zero, 0.f);
    dst[li] = pos < n ? src[(size_t)sidx * n * D + i] : zero;
  }
}
template <typename T>
void launch_pack_k(hipStream_t s, const T* src, T* dst, int S, int n, int n_pad, int D) {
  size_t per = (size_t)n_pad * D;
  hipLaunchKernelGGL(k_pack_k<T>, dim3((unsigned)((per + 255) / 256), S), dim3(256), 0, s, src, dst, n, n_pad, D, 0);
}
template <typename T>
void launch_unpack_k(hipStream_t s, const T* src, T* dst, int S, int n, int n_pad, int D) {
  size_t per = (size_t)n_pad * D;
  hipLaunchKernelGGL(k_pack_k<T>, dim3((unsigned)((per + 255) / 256), S), dim3(256), 0, s, src, dst, n, n_pad, D, 1);
}
template <typename T>
void launch_pack_v(hipStream_t s, const T* src, T* dst, int S, int n, int n_pad, int D) {
  size_t per = (size_t)n_pad * D;
  hipLaunchKernelGGL(k_pack_v<T>, dim3((unsigned)((per + 255) / 256), S), dim3(256), 0, s, src, dst, n, n_pad, D, 0);
}
template <typename T>
void launch_unpack_v(hipStream_t s, const T* src, T* dst, int S, int n, int n_pad, int D) {
  size_t per = (size_t)n_pad * D;
  hipLaunchKernelGGL(k_pack_v<T>, dim3((unsigned)((per + 255) / 256), S), dim3(256), 0, s, src, dst, n, n_pad, D, 1);
}
template void launch_pack_k<float>(hipStream_t, const float*, float*, int, int, int, int);
template void launch_pack_k<bf16_t>(hipStream_t, const bf16_t*, bf16_t*, int, int, int, int);
template void launch_pack_v<float>(hipStream_t, const float*, float*, int, int, int, int);
template void launch_pack_v<bf16_t>(hipStream_t, const bf16_t*, bf16_t*, int, int, int, int);
template void launch_unpack_v<float>(hipStream_t, const float*, float*, int, int, int, int);
template void launch_unpack_v<bf16_t>(hipStream_t, const bf16_t*, bf16_t*, int, int, int, int);
template void launch_pack_k<fp8_t>(hipStream_t, const fp8_t*, fp8_t*, int, int, int, int);
template void launch_pack_v<fp8_t>(hipStream_t, const fp8_t*, fp8_t*, int, int, int, int);
template void launch_unpack_v<fp8_t>(hipStream_t, const fp8_t*, fp8_t*, int, int, int, int);
template void launch_unpack_k<float>(hipStream_t, const float*, float*, int, int, int, int);
template void launch_unpack_k<bf16_t>(hipStream_t, const bf16_t*, bf16_t*, int, int, int, int);
template void launch_unpack_k<fp8_t>(hipStream_t, const fp8_t*, fp8_t*, int, int, int, int);

}  // namespace plt
