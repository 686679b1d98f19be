// Low-bit projections on gfx950's block-scaled matrix cores: c[M,N] (float) = a[M,K] * w[N,K]^T with
//   w in MXFP4: elements e2m1 (4 bits), one power-of-two scale (e8m0 byte) per 32 consecutive k
//   a in MXFP8: elements e4m3 (8 bits), one power-of-two scale per 32 consecutive k
// the reading taken for the "W4A8 quantization of linear layers" of the paper's serving recipe
// [inference efficiency evaluation recipe]: the OCP microscaling formats, which this part's
// v_mfma_scale_f32_16x16x128_f8f6f4 consumes directly (block scales applied inside the instruction).
//
// Quantisation of a block of 32 values v: e = floor(log2(max |v|)) - emax (emax = 2 for e2m1, 8 for e4m3;
// an all-zero block: -127), stored as the byte e + 127; elements = v * 2^-e rounded to the element
// format, nearest even, saturating (6 / 448).
//
// Operand layout of the instruction (measured with one-hot operands): lane = 16 g + m.
//   A (e2m1): lane holds row m, its 32 nibbles (16 bytes, low nibble first) are k = 32 g .. 32 g + 31
//   B (e4m3): lane holds row m, bytes 0..15 are k = 16 g .. 16 g + 15 and bytes 16..31 are k = 64 + 16 g ..
//   scales  : lane (m, g) supplies the scale of row m, k block g (k = 32 g .. 32 g + 31), for both operands;
//             op_sel picks one of the four bytes of the scale register
//   C       : lane holds C[A row 4 g + c][B row m], c = 0..3
// Weights are the A operand (so a lane ends with 4 consecutive output columns of one activation row).
//
// Memory layout.  Weight codes: [strip of 16 rows][chunk of 128 k][lane][16 bytes] -- one wavefront load per
// MFMA is one contiguous KiB, a strip one contiguous stream.  Weight scales: [strip][group of 4 chunks][lane]
// [4 bytes] (byte c = chunk 4*group + c).  Activation codes: row-major [M][K].  Activation scales:
// [M][ceil(K/512)][g][c]: byte (g, c) of group q is the scale of k block 16 q + 4 c + g.
#include "plt_internal.h"
#include <type_traits>

namespace plt {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;

// ---------------------------------------------------------------------------------------------- quantisers
// e2m1 code of v (|v| < 8 after block scaling): nearest value of {0, .5, 1, 1.5, 2, 3, 4, 6}, ties to the
// even code, saturating
__device__ inline unsigned f32_to_e2m1(float v) {
  const float a = fabsf(v);
  unsigned c = a <= 0.25f ? 0u : a < 0.75f ? 1u : a <= 1.25f ? 2u : a < 1.75f ? 3u : a <= 2.5f ? 4u : a < 3.5f ? 5u : a <= 5.0f ? 6u : 7u;
  return c | (v < 0.f ? 8u : 0u);
}

// one thread per (weight row n, k block b): 32 bf16 values in, 16 code bytes (one lane's MFMA operand) and
// one scale byte out, both at their place in the tiled layout
__global__ __launch_bounds__(256) void k_mx_quant_w(const bf16_t* __restrict__ w, uint8_t* __restrict__ codes,
                                                    uint8_t* __restrict__ scales, int N, int K) {
  const int nb = K >> 5;
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)N * nb) return;
  const int n = (int)(t / nb), b = (int)(t - (size_t)n * nb);
  const uint4* src = reinterpret_cast<const uint4*>(w + (size_t)n * K + b * 32);
  float v[32];
  float amax = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint4 u = src[i];
    const unsigned x[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      v[i * 8 + 2 * j] = bf16_to_f32((bf16_t)(x[j] & 0xffffu));
      v[i * 8 + 2 * j + 1] = bf16_to_f32((bf16_t)(x[j] >> 16));
    }
  }
#pragma unroll
  for (int i = 0; i < 32; ++i) amax = fmaxf(amax, fabsf(v[i]));
  const int e = mx_block_exponent(amax, 2);
  unsigned out[4] = {0, 0, 0, 0};
#pragma unroll
  for (int i = 0; i < 32; ++i) out[i >> 3] |= f32_to_e2m1(ldexpf(v[i], -e)) << (4 * (i & 7));
  *reinterpret_cast<uint4*>(codes + mx_wcode_index(n, b * 32, K)) = make_uint4(out[0], out[1], out[2], out[3]);
  scales[mx_wscale_index(n, b, K)] = (uint8_t)(e + 127);
}

// one thread per (activation row, k block): 32 values in, 32 e4m3 bytes (row-major) and one scale byte out.
// Groups of scale bytes beyond K (K not a multiple of 512) are written as 0 by the threads of the last block.
template <typename T>
__global__ __launch_bounds__(256) void k_mx_quant_a(const T* __restrict__ a, uint8_t* __restrict__ codes,
                                                    uint8_t* __restrict__ scales, int M, int K) {
  const int nb = K >> 5, nbp = mx_ascale_row_bytes(K);
  const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (size_t)M * nb) return;
  const int r = (int)(t / nb), b = (int)(t - (size_t)r * nb);
  const T* src = a + (size_t)r * K + b * 32;
  float v[32];
  float amax = 0.f;
#pragma unroll
  for (int i = 0; i < 32; ++i) { v[i] = ld<T>(src + i); amax = fmaxf(amax, fabsf(v[i])); }
  const int e = mx_block_exponent(amax, 8);
  unsigned out[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) out[i] = mx_pack4_e4m3(v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3], e);
  uint4* dst = reinterpret_cast<uint4*>(codes + (size_t)r * K + b * 32);
  dst[0] = make_uint4(out[0], out[1], out[2], out[3]);
  dst[1] = make_uint4(out[4], out[5], out[6], out[7]);
  scales[(size_t)r * nbp + mx_ascale_index(b)] = (uint8_t)(e + 127);
  if (b == nb - 1)
    for (int x = nb; x < nbp; ++x) scales[(size_t)r * nbp + mx_ascale_index(x)] = 0;
}

void launch_mx_quant_w(hipStream_t s, const bf16_t* w, uint8_t* codes, uint8_t* scales, int N, int K) {
  const size_t n = (size_t)N * (K >> 5);
  hipLaunchKernelGGL(k_mx_quant_w, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, w, codes, scales, N, K);
}
template <typename T>
void launch_mx_quant_a(hipStream_t s, const T* a, uint8_t* codes, uint8_t* scales, int M, int K) {
  const size_t n = (size_t)M * (K >> 5);
  hipLaunchKernelGGL(k_mx_quant_a<T>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a, codes, scales, M, K);
}
template void launch_mx_quant_a<float>(hipStream_t, const float*, uint8_t*, uint8_t*, int, int);
template void launch_mx_quant_a<bf16_t>(hipStream_t, const bf16_t*, uint8_t*, uint8_t*, int, int);

// ---------------------------------------------------------------------------------------------- GEMM
// Weight streaming, as the bf16 decode GEMM: a workgroup keeps the activation slice of one K range of 1024
// (up to 128 rows x 1 KiB of e4m3 codes plus their scales) in LDS; its 4 waves walk over groups of NB
// 16-column weight strips whose codes go from HBM straight into registers (one KiB per wavefront load),
// half a K range at a time, the next half prefetched while the current one is multiplied.  One B fragment
// read from LDS feeds NB MFMAs.  Each K range writes its own float slab; consumers add the slabs in a
// fixed order.

template <int MT, int NB>
__global__ __launch_bounds__(256) void k_gemm_mx(const uint8_t* __restrict__ a, const uint8_t* __restrict__ a_sc,
                                                 const uint8_t* __restrict__ w, const uint8_t* __restrict__ w_sc,
                                                 float* __restrict__ c, int M, int N, int K, int n_groups) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds_mx[];   // [MT*16][MX_LDA] codes, then [MT*16][MX_SB] scales
  uint8_t* As = lds_mx;
  uint8_t* Ss = lds_mx + MT * 16 * MX_LDA;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, m16 = lane & 15, g = lane >> 4;
  const int ng = blockIdx.x, rb = blockIdx.y, rng = blockIdx.z;
  const int row0 = rb * (MT * 16);
  const int k0 = rng * MX_KR;
  const int kr = (K - k0 < MX_KR) ? K - k0 : MX_KR;          // valid width of this K range (multiple of 128)
  const int n_chunks = K >> 7;                               // 128-wide chunks per weight row
  const int n_cgrp = (n_chunks + 3) >> 2;                    // groups of 4 chunks (scale dwords) per strip
  const int n_strips = N >> 4, n_grp = (n_strips + NB - 1) / NB;
  const int stride = n_groups * 4;

  struct WBuf { uint4 q[NB][4]; unsigned sc[NB]; };
  WBuf bufA, bufB;
  // half h (0, 1) of this K range for the NB strips of group grp: 4 chunks of codes + their scale dword
  auto wload = [&](WBuf& f, int grp, int h) {
#pragma unroll
    for (int sb = 0; sb < NB; ++sb) {
      int strip = grp * NB + sb; if (strip >= n_strips) strip = n_strips - 1;     // ragged N: a valid strip (stores are masked)
      const int cg = (k0 >> 9) + h;                                                 // chunk group of this half
      const uint8_t* wp = w + ((size_t)strip * n_chunks) * 1024 + lane * 16;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        int ch = cg * 4 + kk; if (ch >= n_chunks) ch = 0;                           // beyond K: an in-range chunk (meets zero codes)
        f.q[sb][kk] = *reinterpret_cast<const uint4*>(wp + (size_t)ch * 1024);
      }
      const int cgs = cg < n_cgrp ? cg : n_cgrp - 1;                                // beyond K: any finite scale will do
      f.sc[sb] = *reinterpret_cast<const unsigned*>(w_sc + (((size_t)strip * n_cgrp + cgs) * 64 + lane) * 4);
    }
  };
  int grp = ng * 4 + wv;
  if (grp < n_grp) wload(bufA, grp, 0);

  // activation slice -> LDS: codes by direct-to-LDS loads (one row = one KiB = one wavefront load), rows beyond M
  // repeat row M-1 (never stored); a ragged range is zero-filled beyond K
  const unsigned lds_as = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)As;
  if (kr == MX_KR) {
    for (int row = wv; row < MT * 16; row += 4) {
      int gm = row0 + row; if (gm >= M) gm = M - 1;
      const uint8_t* src = a + (size_t)gm * K + k0 + lane * 16;
      const unsigned dst = __builtin_amdgcn_readfirstlane(lds_as + (unsigned)row * MX_LDA);
      unsigned keep_m0;                                            // m0 is left as it was found
      asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                   : "=&s"(keep_m0) : "s"(dst), "v"(src) : "memory");
    }
  } else {
    for (int ch = tid; ch < MT * 16 * (MX_KR / 16); ch += 256) {
      const int row = ch / (MX_KR / 16), kc = (ch % (MX_KR / 16)) * 16;
      int gm = row0 + row; if (gm >= M) gm = M - 1;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (kc < kr) v = *reinterpret_cast<const uint4*>(a + (size_t)gm * K + k0 + kc);
      *reinterpret_cast<uint4*>(&As[row * MX_LDA + kc]) = v;
    }
  }
  {
    const int asb = mx_ascale_row_bytes(K);                        // scale bytes per activation row (multiple of 16)
    for (int ch = tid; ch < MT * 16 * 2; ch += 256) {              // two 16-byte scale groups per row and range
      const int row = ch >> 1, h = ch & 1;
      int gm = row0 + row; if (gm >= M) gm = M - 1;
      const int cg = (k0 >> 9) + h;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (cg * 16 < asb) v = *reinterpret_cast<const uint4*>(a_sc + (size_t)gm * asb + cg * 16);
      *reinterpret_cast<uint4*>(&Ss[row * MX_SB + h * 16]) = v;
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  f32x4 acc[NB][MT];
  struct BFrag { uint4 lo, hi; };
  auto bload = [&](int h, int idx) {           // fragment idx = kk * MT + i of half h
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
    for (int idx = 0; idx < 4 * MT; ++idx) {   // the next fragment is requested before the current one is multiplied
      const int kk = idx / MT, i = idx - kk * MT;
      BFrag nxt = cur;
      if (idx + 1 < 4 * MT) nxt = bload(h, idx + 1);
      const i32x8 bv = {(int)cur.lo.x, (int)cur.lo.y, (int)cur.lo.z, (int)cur.lo.w, (int)cur.hi.x, (int)cur.hi.y, (int)cur.hi.z, (int)cur.hi.w};
#pragma unroll
      for (int sb = 0; sb < NB; ++sb) {
        const i32x8 av = {(int)f.q[sb][kk].x, (int)f.q[sb][kk].y, (int)f.q[sb][kk].z, (int)f.q[sb][kk].w, 0, 0, 0, 0};
        // cbsz 4: A is e2m1; blgp 0: B is e4m3; op_sel kk: byte kk of the scale registers
        if (kk == 0) acc[sb][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, acc[sb][i], 4, 0, 0, (int)f.sc[sb], 0, (int)bsc[i]);
        else if (kk == 1) acc[sb][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, acc[sb][i], 4, 0, 1, (int)f.sc[sb], 1, (int)bsc[i]);
        else if (kk == 2) acc[sb][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, acc[sb][i], 4, 0, 2, (int)f.sc[sb], 2, (int)bsc[i]);
        else acc[sb][i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, acc[sb][i], 4, 0, 3, (int)f.sc[sb], 3, (int)bsc[i]);
      }
      cur = nxt;
      __builtin_amdgcn_sched_barrier(0);       // keeps later fragment reads from being hoisted up here (register pressure)
    }
  };
  float* cs = c + (size_t)rng * M * N;
  for (; grp < n_grp; grp += stride) {
    // the activation fragments are the same for every strip group: without this the compiler reads them all
    // from LDS once, ahead of the loop, and keeps them in (more than the available) registers
    asm volatile("" ::: "memory");
#pragma unroll
    for (int sb = 0; sb < NB; ++sb)
#pragma unroll
      for (int i = 0; i < MT; ++i) acc[sb][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    wload(bufB, grp, 1);
    mac(bufA, 0);
    // next group's first half; past the last group the same group is loaded again (in bounds, unused): a
    // branch here would split the block, and the compiler would move the first half's MFMAs below it
    wload(bufA, grp + stride < n_grp ? grp + stride : grp, 0);
    mac(bufB, 1);
    // the results are needed whether or not a row is stored: without this the compiler moves every MFMA down
    // into the conditional store of its row tile and keeps all activation fragments alive until then
#pragma unroll
    for (int sb = 0; sb < NB; ++sb)
#pragma unroll
      for (int i = 0; i < MT; ++i) asm volatile("" : "+v"(acc[sb][i]));
    // acc[sb][i][e] = C[row0 + i*16 + m16][(grp*NB + sb)*16 + 4*g + e]
#pragma unroll
    for (int sb = 0; sb < NB; ++sb) {
      const int gn = (grp * NB + sb) * 16 + 4 * g;
      if (gn >= N) continue;
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int gm = row0 + i * 16 + m16;
        if (gm < M) *reinterpret_cast<f32x4*>(cs + (size_t)gm * N + gn) = acc[sb][i];
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------- prefill-sized row counts
// The same product for thousands of rows (matrix-core-bound): workgroup tile 256 rows x 256 columns, whole K (no
// split-K slabs), K in steps of one 128-wide chunk through two LDS stages filled HBM -> LDS directly; 8 waves as
// 2 x 4, each 128 rows x 64 columns = 8 x 4 tiles of the block-scaled MFMA.  A stage holds the activation tile
// (256 rows x 128 code bytes; the 16-byte pieces of a row XOR-swizzled with the row number so that the fragment
// reads of 16 rows touch every bank once) and 16 weight strips x 1 KiB exactly as they lie in memory (that IS the
// A-operand layout: lane l reads bytes 16 l ..).  The block scales go from memory straight into registers, one
// dword per lane and 4 chunks (512 k) for either operand, fetched one group of 4 chunks ahead.
__global__ __launch_bounds__(512) void k_gemm_mx_tile(const uint8_t* __restrict__ a, const uint8_t* __restrict__ a_sc,
                                                      const uint8_t* __restrict__ w, const uint8_t* __restrict__ w_sc,
                                                      float* __restrict__ c, int M, int N, int K) {
  constexpr int BM = 256, BN = 256, THREADS = 512, WN = 4, MI = 8, NT = 4;
  constexpr int A_BYTES = BM * 128, W_BYTES = (BN / 16) * 1024, STAGE_BYTES = A_BYTES + W_BYTES;
  extern __shared__ __attribute__((aligned(16))) char mxt_lds[];
  // The 128 accumulators and the 8-register operand tuples leave little room: what is the same for a whole wave
  // is kept in scalar registers (hence the readfirstlane), and per-lane addresses as 32-bit offsets from them.
  const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), m16 = lane & 15, g = lane >> 4;
  const int wm = wv / WN, wn = wv % WN;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int n_chunks = K >> 7, n_cgrp = (n_chunks + 3) >> 2, n_strips = N >> 4, asb = mx_ascale_row_bytes(K);
  // this thread's pieces of a stage: 4 of the activation tile (slot s = i*THREADS + tid -> row s/8, piece (s%8) ^ (row%8)),
  // 2 of the weight strips (slot s -> strip s/64 of the tile, byte 16 (s%64) of its KiB)
  unsigned pa[4];                       // byte offsets into a (M * K < 2^32)
  const uint8_t* pw[2];                 // the two strips are the same for the whole wave: scalar base + 16 lane
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int sl = i * THREADS + tid, row = sl >> 3, pc = (sl & 7) ^ (row & 7);
    int gm = m0 + row; if (gm >= M) gm = M - 1;                 // rows beyond M: computed, never stored
    pa[i] = (unsigned)gm * (unsigned)K + pc * 16;
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    int strip = (n0 >> 4) + i * 8 + wv; if (strip >= n_strips) strip = n_strips - 1;      // slot (i*512 + tid) / 64 = 8 i + wave
    pw[i] = w + (size_t)strip * n_chunks * 1024;
  }
  const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)mxt_lds;
  auto dma16 = [](const uint8_t* src, unsigned lds_wave_base) {  // lane l: 16 bytes -> LDS[lds_wave_base + 16 l]
    unsigned keep_m0;                                            // m0 is left as it was found
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep_m0) : "s"(lds_wave_base), "v"(src) : "memory");
  };
  auto issue = [&](int ch) {                                     // chunk ch -> stage ch & 1
    const unsigned stage = lds0 + (unsigned)(ch & 1) * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      dma16(a + ((size_t)pa[i] + (size_t)ch * 128), stage + (unsigned)(i * THREADS + wv * 64) * 16);
#pragma unroll
    for (int i = 0; i < 2; ++i)
      dma16(pw[i] + (size_t)ch * 1024 + lane * 16, stage + A_BYTES + (unsigned)(i * THREADS + wv * 64) * 16);
  };
  // scale dwords of chunk group q: weights: strip j of this wave, this lane; activations: row tile i, this lane's row, block g
  const uint8_t* wsp[NT];               // per wave (scalar); + 4 lane
  unsigned asp[MI];                     // byte offsets into a_sc
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    int strip = (n0 >> 4) + wn * NT + j; if (strip >= n_strips) strip = n_strips - 1;
    wsp[j] = w_sc + (size_t)strip * n_cgrp * 256;
  }
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    int gm = m0 + wm * 128 + i * 16 + m16; if (gm >= M) gm = M - 1;
    asp[i] = (unsigned)gm * (unsigned)asb + g * 4;
  }
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
  const int sw0 = (g ^ (m16 & 7)) * 16;                  // byte offset of the lane's first piece inside its row
  // one chunk: kk = its place in the group of 4 (selects the scale byte), compile-time
  auto step = [&](int ch, auto kk_tag) {
    constexpr int kk = decltype(kk_tag)::value;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of chunk ch has landed (and the next group's scales)
    __syncthreads();                                   // ... and everyone's; chunk ch - 1 is no longer read
    if (ch + 1 < n_chunks) issue(ch + 1);
    const char* As = mxt_lds + (ch & 1) * STAGE_BYTES;
    const char* Ws = As + A_BYTES;
    uint4 fw[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) fw[j] = *reinterpret_cast<const uint4*>(Ws + (wn * NT + j) * 1024 + lane * 16);
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
    if (q + 1 < n_cgrp) load_scales(q + 1, wsc_n, asc_n);     // waited for at the top of the next step, a chunk of MFMAs later
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
  // acc[i][j][x]: row m0 + wm*128 + i*16 + m16, column n0 + (wn*NT + j)*16 + 4 g + x
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int gm = m0 + wm * 128 + i * 16 + m16;
    if (gm >= M) continue;
    float* o = c + (size_t)gm * N;
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int gn = n0 + (wn * NT + j) * 16 + 4 * g;
      if (gn < N) *reinterpret_cast<f32x4*>(o + gn) = acc[i][j];          // N % 16 == 0: whole groups of 4 columns
    }
  }
}

// rows from which the tiled kernel takes over (its 256 x 256 tiles must fill the chip)
static bool gemm_mx_tile_applies(int M, int N, int K) {
  const long tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
  return M >= 512 && tiles >= 128 && (K % 128) == 0 && (N % 16) == 0;
}

// number of [M, N] float slabs the product leaves: one per K range of the streaming kernel, a single one from the
// tiled kernel
int gemm_mx_splits(int M, int N, int K) { return gemm_mx_tile_applies(M, N, K) ? 1 : (K + MX_KR - 1) / MX_KR; }

template <int MT, int NB>
static void mx_launch(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const uint8_t* w, const uint8_t* w_sc, float* c,
                      int M, int N, int K) {
  const size_t lds = (size_t)MT * 16 * (MX_LDA + MX_SB);
  // opt-in to more than 64 KB of dynamic LDS: once per template instance, thread-safe (initialisation of a local static)
  static const hipError_t attr_once = hipFuncSetAttribute((const void*)k_gemm_mx<MT, NB>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  (void)attr_once;
  const int S = (K + MX_KR - 1) / MX_KR, rbs = (M + MT * 16 - 1) / (MT * 16);
  const int n_grp = ((N >> 4) + NB - 1) / NB;
  const int per_cu = MT == 8 ? 1 : 2;                         // workgroups that fit a compute unit (LDS)
  int n_groups = 256 * per_cu / (S * (rbs < 4 ? rbs : 4)); if (n_groups < 1) n_groups = 1;
  if (n_groups > (n_grp + 3) / 4) n_groups = (n_grp + 3) / 4;
  hipLaunchKernelGGL((k_gemm_mx<MT, NB>), dim3(n_groups, rbs, S), dim3(256), lds, s, a, a_sc, w, w_sc, c, M, N, K, n_groups);
}

// c: gemm_mx_splits(M, N, K) slabs of [M, N] floats.  N % 16 == 0, K % 128 == 0.  Strips per wave task (NB) grow
// until the waves of one (K range, row block) cover the strips in one pass if possible.
void launch_gemm_mx(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const uint8_t* w, const uint8_t* w_sc, float* c,
                    int M, int N, int K) {
  if (gemm_mx_tile_applies(M, N, K)) {
    constexpr int LDS_BYTES = 2 * (256 * 128 + 16 * 1024);
    // opt-in to more than 64 KB of dynamic LDS: once per template instance, thread-safe (initialisation of a local static)
    static const hipError_t attr_once = hipFuncSetAttribute((const void*)k_gemm_mx_tile, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    (void)attr_once;
    hipLaunchKernelGGL(k_gemm_mx_tile, dim3((N + 255) / 256, (M + 255) / 256), dim3(512), LDS_BYTES, s, a, a_sc, w, w_sc, c, M, N, K);
    return;
  }
  const int n_strips = N >> 4, S = (K + MX_KR - 1) / MX_KR;
  const bool small = M <= 64;
  int slots = 256 * (small ? 2 : 1) / S * 4; if (slots < 4) slots = 4;
  const int nb = (n_strips + slots - 1) / slots;
#define MX_CASE(MT_, NB_) mx_launch<MT_, NB_>(s, a, a_sc, w, w_sc, c, M, N, K)
  if (small) { if (nb >= 3) MX_CASE(4, 4); else if (nb == 2) MX_CASE(4, 2); else MX_CASE(4, 1); }
  else       { if (nb >= 3) MX_CASE(8, 4); else if (nb == 2) MX_CASE(8, 2); else MX_CASE(8, 1); }
#undef MX_CASE
}

}  // namespace plt
