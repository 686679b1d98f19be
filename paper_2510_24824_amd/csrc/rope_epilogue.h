// S3 of a layer (rotary embedding, gate logit on the un-rotated query [Eq. 2], cache appends [Alg. 1 l.5-7,
// Alg. 3 l.1, l.4]) as the epilogue of a QKV product that leaves its result in matrix-core accumulators: shared by
// the bf16 tile kernel and the low-bit row-tile kernel, whose accumulator layouts agree (lane (m16, g) of a wave
// holds, for row tile i and 16-column tile j, row 16 i + m16 and columns 16 j + 4 g .. 4 g + 3).
#pragma once
#include "plt_internal.h"

namespace plt {

typedef __attribute__((ext_vector_type(4))) float f32x4;

// What the EPI_ROPE epilogue needs beyond the product: row gm of the chunk is position gm % n of chunk sequence gm / n
struct RopeEpi {
  const float* gate_w; const float* gate_b; const double* inv_freq;
  bf16_t* q_out; float* z_out;
  KvView kv;
  int n, loop, Hq, Hkv, mode;
  const int32_t* pos; int L;      // EPI_ROPE_DEC: row gm is loop stage gm % L of sequence gm / L at position pos[gm / L]
};

// four consecutive cache elements from four floats (destination aligned to the four)
__device__ inline void store4(bf16_t* dst, const f32x4 v) { *reinterpret_cast<bf16x4*>(dst) = __builtin_convertvector(v, bf16x4); }
__device__ inline void store4(fp8_t* dst, const f32x4 v) {
  float c[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) c[e] = fminf(fmaxf(v[e], -448.f), 448.f);
  const int pk = __builtin_amdgcn_cvt_pk_fp8_f32(c[0], c[1], 0, false);
  *reinterpret_cast<unsigned*>(dst) = (unsigned)__builtin_amdgcn_cvt_pk_fp8_f32(c[2], c[3], pk, true);
}

// S3 of the layer on a wave's accumulators: acc[i][j][e] = row row0 + 16 i + m16, column col0 + 16 j + 4 g + e of
// the QKV product; the wave's NT*16 columns are whole heads of D.  Same arithmetic as k_rope_append_tile: angle in
// turns reduced in double, hardware sine / cosine, pairs (f, f + D/2); the gate logit from the un-rotated query;
// first-loop K/V into the shared cache, later loops' into the chunk's own K/V and (last w positions) the rings.
template <int D, typename KT, int MI, int NT>
__device__ inline void rope_epilogue(f32x4 (&acc)[MI][NT], const RopeEpi& ep, int row0, int col0, int M, int N, int m16, int g) {
  constexpr int HT = D / 16, PT = HT / 2, half = D / 2;     // 16-column tiles per head, per rotation half
  static_assert((NT * 16) % D == 0, "a wave holds whole heads");
  const int Hq = ep.Hq, Hkv = ep.Hkv, n = ep.n, mode = ep.mode, loop = ep.loop;
  const KvView& kv = ep.kv;
#pragma unroll
  for (int hh = 0; hh < NT / HT; ++hh) {
    const int c0 = col0 + hh * D;
    if (c0 >= N) break;                                      // (the same for the whole wave)
    const int hs = c0 / D;
    const bool is_q = hs < Hq, is_k = !is_q && hs < Hq + Hkv;
    const bool want_z = is_q && mode == 0 && loop > 0;
    double fr[PT][4];
    float gw_lo[PT][4], gw_hi[PT][4];
    if (is_q || is_k) {
#pragma unroll
      for (int t = 0; t < PT; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e) fr[t][e] = ep.inv_freq[16 * t + 4 * g + e] * 0.15915494309189535;
    }
    if (want_z) {
#pragma unroll
      for (int t = 0; t < PT; ++t) {
        const float4 a = *reinterpret_cast<const float4*>(ep.gate_w + hs * D + 16 * t + 4 * g);
        const float4 b = *reinterpret_cast<const float4*>(ep.gate_w + hs * D + half + 16 * t + 4 * g);
        gw_lo[t][0] = a.x; gw_lo[t][1] = a.y; gw_lo[t][2] = a.z; gw_lo[t][3] = a.w;
        gw_hi[t][0] = b.x; gw_hi[t][1] = b.y; gw_hi[t][2] = b.z; gw_hi[t][3] = b.w;
      }
    }
    const int kh = is_k ? hs - Hq : hs - Hq - Hkv;
    const bool own = mode == 0 && loop > 0;                  // non-first loop of the method: own K/V (+ ring tail)
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int gm = row0 + i * 16 + m16;
      const bool ok = gm < M;
      const int b = ok ? gm / n : 0, p = ok ? gm - b * n : 0;
      f32x4* lo = &acc[i][hh * HT];
      f32x4* hi = &acc[i][hh * HT + PT];
      if (want_z) {                                          // gate logit on the un-rotated query [Alg. 3 l.4]
        float zp = 0.f;
#pragma unroll
        for (int t = 0; t < PT; ++t)
#pragma unroll
          for (int e = 0; e < 4; ++e) zp += lo[t][e] * gw_lo[t][e] + hi[t][e] * gw_hi[t][e];
        zp = row4_add_f32(zp);                               // the four lanes that share the row
        if (ok && g == 0) ep.z_out[(size_t)gm * Hq + hs] = zp + ep.gate_b[hs];
      }
      if (is_q || is_k) {
#pragma unroll
        for (int t = 0; t < PT; ++t)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            double a = (double)p * fr[t][e];
            a -= rint(a);
            const float sn = __builtin_amdgcn_sinf((float)a), c = __builtin_amdgcn_cosf((float)a);
            const float l0 = lo[t][e], h0 = hi[t][e];
            lo[t][e] = l0 * c - h0 * sn; hi[t][e] = h0 * c + l0 * sn;
          }
      }
      if (!ok) continue;
      if (is_q) {
        bf16_t* dst = ep.q_out + (size_t)gm * Hq * D + (size_t)hs * D + 4 * g;
#pragma unroll
        for (int t = 0; t < PT; ++t) { store4(dst + 16 * t, lo[t]); store4(dst + half + 16 * t, hi[t]); }
        continue;
      }
      if (mode == 2 && loop > 0) continue;                   // KV-share ablation: non-first loops keep no K/V
      const size_t stream = own ? (size_t)b * Hkv + kh : (size_t)(kv.b0 + b) * Hkv + kh;
      const size_t stream_elems = (size_t)(own ? kv.n_pad_loc : kv.n_pad) * D;
      const bool ring = own && p >= n - kv.w;                // the w most recent entries also enter the ring
      const int slot = p % kv.w;
      const size_t rstream = (((size_t)(kv.b0 + b) * kv.n_rings + (loop - 1)) * Hkv + kh) * (size_t)kv.w_pad * D;
      if (is_k) {
        KT* dst = (KT*)(own ? kv.k_loc : kv.k_share) + stream * stream_elems;
#pragma unroll
        for (int t = 0; t < PT; ++t) {
          store4(dst + kblk_index<KT>(p, 16 * t + 4 * g, D), lo[t]);
          store4(dst + kblk_index<KT>(p, half + 16 * t + 4 * g, D), hi[t]);
        }
        if (ring) {
          KT* rd = (KT*)kv.k_ring + rstream;
#pragma unroll
          for (int t = 0; t < PT; ++t) {
            store4(rd + kblk_index<KT>(slot, 16 * t + 4 * g, D), lo[t]);
            store4(rd + kblk_index<KT>(slot, half + 16 * t + 4 * g, D), hi[t]);
          }
        }
      } else {
        // V is stored position-fastest: a lane's four features of one position are four separate elements; the 16
        // lanes of a row group write 16 consecutive positions of a feature, i.e. whole 16-byte chunks per instruction
        KT* dst = (KT*)(own ? kv.v_loc : kv.v_share) + stream * stream_elems;
#pragma unroll
        for (int t = 0; t < HT; ++t)
#pragma unroll
          for (int e = 0; e < 4; ++e) st<KT>(dst + vblk_index<KT>(p, 16 * t + 4 * g + e, D), lo[t][e]);
        if (ring) {
          KT* rd = (KT*)kv.v_ring + rstream;
#pragma unroll
          for (int t = 0; t < HT; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) st<KT>(rd + vblk_index<KT>(slot, 16 * t + 4 * g + e, D), lo[t][e]);
        }
      }
    }
  }
}

// S3 for the rows of a decode step: as rope_epilogue, but every row carries its own loop stage and position (row gm =
// stage gm % L of sequence gm / L at position pos[gm / L]), the first stage appends to the shared cache (the cache of
// its stage in the per-loop-cache mode), later stages to their ring slot p mod w.  Same arithmetic as k_rope_append.
template <int D, typename KT, int MI, int NT>
__device__ inline void rope_epilogue_decode(f32x4 (&acc)[MI][NT], const RopeEpi& ep, int row0, int col0, int M, int N, int m16, int g) {
  constexpr int HT = D / 16, PT = HT / 2, half = D / 2;
  static_assert((NT * 16) % D == 0, "a wave holds whole heads");
  const int Hq = ep.Hq, Hkv = ep.Hkv, L = ep.L, mode = ep.mode;
  const KvView& kv = ep.kv;
#pragma unroll
  for (int hh = 0; hh < NT / HT; ++hh) {
    const int c0 = col0 + hh * D;
    if (c0 >= N) break;                                      // (the same for the whole wave)
    const int hs = c0 / D;
    const bool is_q = hs < Hq, is_k = !is_q && hs < Hq + Hkv;
    const bool want_z = is_q && mode == 0 && L > 1;
    double fr[PT][4];
    float gw_lo[PT][4], gw_hi[PT][4];
    if (is_q || is_k) {
#pragma unroll
      for (int t = 0; t < PT; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e) fr[t][e] = ep.inv_freq[16 * t + 4 * g + e] * 0.15915494309189535;
    }
    if (want_z) {
#pragma unroll
      for (int t = 0; t < PT; ++t) {
        const float4 a = *reinterpret_cast<const float4*>(ep.gate_w + hs * D + 16 * t + 4 * g);
        const float4 b = *reinterpret_cast<const float4*>(ep.gate_w + hs * D + half + 16 * t + 4 * g);
        gw_lo[t][0] = a.x; gw_lo[t][1] = a.y; gw_lo[t][2] = a.z; gw_lo[t][3] = a.w;
        gw_hi[t][0] = b.x; gw_hi[t][1] = b.y; gw_hi[t][2] = b.z; gw_hi[t][3] = b.w;
      }
    }
    const int kh = is_k ? hs - Hq : hs - Hq - Hkv;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int gm = row0 + i * 16 + m16;
      const bool ok = gm < M;
      const int b = ok ? gm / L : 0, l = ok ? gm - b * L : 0, p = ok ? ep.pos[b] : 0;
      f32x4* lo = &acc[i][hh * HT];
      f32x4* hi = &acc[i][hh * HT + PT];
      if (want_z) {                                          // gate logit on the un-rotated query [Alg. 3 l.4]
        float zp = 0.f;
#pragma unroll
        for (int t = 0; t < PT; ++t)
#pragma unroll
          for (int e = 0; e < 4; ++e) zp += lo[t][e] * gw_lo[t][e] + hi[t][e] * gw_hi[t][e];
        zp = row4_add_f32(zp);                               // the four lanes that share the row
        if (ok && l > 0 && g == 0) ep.z_out[((size_t)b * (L - 1) + (l - 1)) * Hq + hs] = zp + ep.gate_b[hs];
      }
      if (is_q || is_k) {
#pragma unroll
        for (int t = 0; t < PT; ++t)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            double a = (double)p * fr[t][e];
            a -= rint(a);
            const float sn = __builtin_amdgcn_sinf((float)a), c = __builtin_amdgcn_cosf((float)a);
            const float l0 = lo[t][e], h0 = hi[t][e];
            lo[t][e] = l0 * c - h0 * sn; hi[t][e] = h0 * c + l0 * sn;
          }
      }
      if (!ok) continue;
      if (is_q) {
        bf16_t* dst = ep.q_out + (size_t)gm * Hq * D + (size_t)hs * D + 4 * g;
#pragma unroll
        for (int t = 0; t < PT; ++t) { store4(dst + 16 * t, lo[t]); store4(dst + half + 16 * t, hi[t]); }
        continue;
      }
      if (mode == 2 && l > 0) continue;                      // KV-share ablation: non-first loops keep no K/V
      const int bg = kv.b0 + b;
      KT *kd, *vd; int at;
      if (mode != 0 || l == 0) {                             // first loop: the shared cache [Sec. 2.2.2]
        const size_t off = (mode == 3 ? (size_t)l * kv.cache_stride : 0) + ((size_t)bg * Hkv + kh) * (size_t)kv.n_pad * D;
        kd = (KT*)kv.k_share + off; vd = (KT*)kv.v_share + off; at = p;
      } else {                                               // later loops: only the w most recent entries survive
        const size_t off = (((size_t)bg * kv.n_rings + (l - 1)) * Hkv + kh) * (size_t)kv.w_pad * D;
        kd = (KT*)kv.k_ring + off; vd = (KT*)kv.v_ring + off; at = p % kv.w;
      }
      if (is_k) {
#pragma unroll
        for (int t = 0; t < PT; ++t) {
          store4(kd + kblk_index<KT>(at, 16 * t + 4 * g, D), lo[t]);
          store4(kd + kblk_index<KT>(at, half + 16 * t + 4 * g, D), hi[t]);
        }
      } else {
#pragma unroll
        for (int t = 0; t < HT; ++t)
#pragma unroll
          for (int e = 0; e < 4; ++e) st<KT>(vd + vblk_index<KT>(at, 16 * t + 4 * g + e, D), lo[t][e]);
      }
    }
  }
}

}  // namespace plt
