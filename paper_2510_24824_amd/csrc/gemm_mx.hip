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
#include "rope_epilogue.h"
#include <type_traits>

namespace plt {

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

// ---------------------------------------------------------------------------------------------- decode-sized row counts
// The same product for the few hundred rows of a decode step, organised like the bf16 row tiles: a workgroup takes
// BM rows x 64 columns (4 weight strips) x one run of K (blockIdx.z; runs are whole
// groups of 4 chunks, so that a scale dword never straddles two runs) and writes one float slab per run.  Chunks of
// 128 k go HBM -> LDS directly through a ring of STAGES stages: the activation rows (BM x 128 code bytes, 16-byte
// pieces XOR-swizzled with the row number) and the 4 strips' KiB as they lie in memory; only the oldest chunk in
// flight is waited for (loads return in order), one bare barrier per chunk.  4 waves, each BM / 4 rows x all 64
// columns.  The block scales (one dword per lane and group of 4 chunks) come the same way, a group ahead.
// EPI 1 (gate/up): the tile is 32 gate + the matching 32 up columns over the whole K, and its epilogue applies SwiGLU
// and quantises the 32 hidden values of a row - exactly one block - to e4m3 with their scale byte: no slabs and no
// separate activation kernel.
enum { MXR_F32 = 0, MXR_SWIGLU = 1, MXR_ROPE = 2 };
template <int EPI, int BM, int STAGES, int NT = 4, int D = 128, typename KT = bf16_t>
__global__ __launch_bounds__(256) void k_gemm_mx_rows(const uint8_t* __restrict__ a, const uint8_t* __restrict__ a_sc,
                                                      const uint8_t* __restrict__ w, const uint8_t* __restrict__ w_sc,
                                                      void* __restrict__ out, uint8_t* __restrict__ out_sc, int M, int N, int K,
                                                      const RopeEpi ep) {
  // N: MXR_F32 / MXR_ROPE: output columns (= rows of w); MXR_SWIGLU: F (w has 2F rows: gate rows, then up rows; the output F columns)
  // NT: 16-column weight strips per tile (4; 8 for MXR_ROPE, whose waves must hold whole heads)
  constexpr int THREADS = 256, MI = BM / 64, DMA_A = BM * 8 / THREADS, DMA_W = NT / 4, DMA_N = DMA_A + DMA_W;
  constexpr int A_BYTES = BM * 128, STAGE_BYTES = A_BYTES + NT * 1024;
  static_assert((BM == 64 || BM == 128 || BM == 256) && (NT == 4 || NT == 8) && (EPI != MXR_SWIGLU || NT == 4), "tile shape");
  extern __shared__ __attribute__((aligned(16))) char mxr_lds[];
  const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6), m16 = lane & 15, g = lane >> 4;
  const int m0 = blockIdx.y * BM, tile_n = blockIdx.x;
  const int n_chunks = K >> 7, n_cgrp = (n_chunks + 3) >> 2, asb = mx_ascale_row_bytes(K);
  const int w_rows = EPI == MXR_SWIGLU ? 2 * N : N, n_strips = w_rows >> 4;
  // weight strip behind tile strip j (beyond the matrix: clamped, never stored)
  auto strip_of = [&](int j) -> int {
    int st = EPI == MXR_SWIGLU ? (j < 2 ? tile_n * 2 + j : (N >> 4) + tile_n * 2 + (j - 2)) : tile_n * NT + j;
    return st < n_strips ? st : n_strips - 1;
  };
  // this workgroup's run of chunk groups
  const int gpz = (n_cgrp + (int)gridDim.z - 1) / (int)gridDim.z;
  const int q0 = (int)blockIdx.z * gpz, q1 = q0 + gpz < n_cgrp ? q0 + gpz : n_cgrp;
  const int ch0 = q0 * 4, ch1 = q1 * 4 < n_chunks ? q1 * 4 : n_chunks;              // (an empty run writes a slab of zeros)
  // this thread's pieces of a stage: slot s = i*THREADS + tid -> row s/8, piece (s%8) ^ (row%8); one weight strip per wave
  unsigned pa[DMA_A];
#pragma unroll
  for (int i = 0; i < DMA_A; ++i) {
    const int sl = i * THREADS + tid, row = sl >> 3, pc = (sl & 7) ^ (row & 7);
    int gm = m0 + row; if (gm >= M) gm = M - 1;                 // rows beyond M: computed, never stored
    pa[i] = (unsigned)gm * (unsigned)K + pc * 16;
  }
  const uint8_t* pw[DMA_W];                                     // wave wv fetches tile strips wv, wv + 4
#pragma unroll
  for (int t = 0; t < DMA_W; ++t) pw[t] = w + (size_t)strip_of(wv + 4 * t) * n_chunks * 1024 + lane * 16;
  const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)mxr_lds;
  auto dma16 = [](const uint8_t* src, unsigned lds_wave_base) {  // lane l: 16 bytes -> LDS[lds_wave_base + 16 l]
    unsigned keep_m0;                                            // m0 is left as it was found
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep_m0) : "s"(lds_wave_base), "v"(src) : "memory");
  };
  auto issue = [&](int ch) {                                     // chunk ch -> stage (ch - ch0) % STAGES
    const unsigned stage = lds0 + (unsigned)((ch - ch0) % STAGES) * STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < DMA_A; ++i)
      dma16(a + ((size_t)pa[i] + (size_t)ch * 128), stage + (unsigned)(i * THREADS + wv * 64) * 16);
#pragma unroll
    for (int t = 0; t < DMA_W; ++t) dma16(pw[t] + (size_t)ch * 1024, stage + A_BYTES + (unsigned)(wv + 4 * t) * 1024);
  };
  // Scale dwords of chunk group q (one per lane covers the group's 4 chunks) take the same road, 4 bytes per lane: wave
  // j fetches strip j's (lane (m, g): weight row m, block g), every wave those of its own row tiles (row m16, block
  // g), into one of two scale areas behind the stages; the registers are filled from there at the group's first chunk
  constexpr int SC_OFF = STAGES * STAGE_BYTES, SC_BYTES = NT * 256 + 4 * MI * 256;
  const uint8_t* wsp[DMA_W];
#pragma unroll
  for (int t = 0; t < DMA_W; ++t) wsp[t] = w_sc + (size_t)strip_of(wv + 4 * t) * n_cgrp * 256 + lane * 4;
  unsigned asp[MI];
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    int gm = m0 + wv * (MI * 16) + i * 16 + m16; if (gm >= M) gm = M - 1;
    asp[i] = (unsigned)gm * (unsigned)asb + g * 4;
  }
  auto dma4 = [](const uint8_t* src, unsigned lds_wave_base) {   // lane l: 4 bytes -> LDS[lds_wave_base + 4 l]
    unsigned keep_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep_m0) : "s"(lds_wave_base), "v"(src) : "memory");
  };
  auto issue_scales = [&](int q) {
    const unsigned area = lds0 + SC_OFF + (unsigned)((q - q0) & 1) * SC_BYTES;
#pragma unroll
    for (int t = 0; t < DMA_W; ++t) dma4(wsp[t] + (size_t)q * 256, area + (unsigned)(wv + 4 * t) * 256);
#pragma unroll
    for (int i = 0; i < MI; ++i) dma4(a_sc + ((size_t)asp[i] + q * 16), area + NT * 256 + (unsigned)(wv * MI + i) * 256);
  };
  unsigned wsc[NT], asc[MI];
  f32x4 acc[MI][NT];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int sw0 = (g ^ (m16 & 7)) * 16;                  // byte offset of the lane's first piece inside its row
  // one chunk: kk = its place in the group of 4 (selects the scale byte), compile-time
  auto step = [&](int ch, auto kk_tag) {
    constexpr int kk = decltype(kk_tag)::value;
    // this wave's part of chunk ch has landed: everything but the STAGES - 2 younger chunks (the scale dwords of a
    // group are requested a group ahead, between two chunks: they are older than what may stay in flight at the
    // group's first chunk)
    if (ch + STAGES - 2 >= ch1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(%0)" :: "n"((STAGES - 2) * DMA_N) : "memory");
    __builtin_amdgcn_s_barrier();                      // ... and everyone's; every wave is done with chunk ch - 1 (bare: the loads in flight stay in flight)
    if (ch + STAGES - 1 < ch1) issue(ch + STAGES - 1);
    else asm volatile("" ::: "memory");
    if constexpr (kk == 0) {
      const int q = ch >> 2;
      if (q + 1 < q1) issue_scales(q + 1);
      const char* sc = mxr_lds + SC_OFF + ((q - q0) & 1) * SC_BYTES;
#pragma unroll
      for (int j = 0; j < NT; ++j) wsc[j] = *reinterpret_cast<const unsigned*>(sc + j * 256 + lane * 4);
#pragma unroll
      for (int i = 0; i < MI; ++i) asc[i] = *reinterpret_cast<const unsigned*>(sc + NT * 256 + (wv * MI + i) * 256 + lane * 4);
    }
    const char* As = mxr_lds + ((ch - ch0) % STAGES) * STAGE_BYTES;
    const char* Ws = As + A_BYTES;
    uint4 fw[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) fw[j] = *reinterpret_cast<const uint4*>(Ws + j * 1024 + lane * 16);
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const char* ap = As + (wv * (MI * 16) + i * 16 + m16) * 128;
      const uint4 lo = *reinterpret_cast<const uint4*>(ap + sw0), hi = *reinterpret_cast<const uint4*>(ap + (sw0 ^ 64));
      const i32x8 bv = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const i32x8 av = {(int)fw[j].x, (int)fw[j].y, (int)fw[j].z, (int)fw[j].w, 0, 0, 0, 0};
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(av, bv, acc[i][j], 4, 0, kk, (int)wsc[j], kk, (int)asc[i]);
      }
    }
  };
  if (q0 < q1) issue_scales(q0);
#pragma unroll
  for (int st = 0; st < STAGES - 1; ++st) if (ch0 + st < ch1) issue(ch0 + st);
  for (int q = q0; q < q1; ++q) {
    const int c4 = q * 4;
    step(c4, std::integral_constant<int, 0>{});
    if (c4 + 1 < ch1) step(c4 + 1, std::integral_constant<int, 1>{});
    if (c4 + 2 < ch1) step(c4 + 2, std::integral_constant<int, 2>{});
    if (c4 + 3 < ch1) step(c4 + 3, std::integral_constant<int, 3>{});
  }
  // acc[i][j][x]: row m0 + wv*MI*16 + i*16 + m16, column 4 g + x of tile strip j
  if constexpr (EPI == MXR_ROPE) {
    rope_epilogue_decode<D, KT, MI, NT>(acc, ep, m0 + wv * (MI * 16), tile_n * (NT * 16), M, N, m16, g);
  } else if constexpr (EPI == MXR_SWIGLU) {
    const int nbp = mx_ascale_row_bytes(N);
    uint8_t* codes = (uint8_t*)out;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int gm = m0 + wv * (MI * 16) + i * 16 + m16;
      float h[2][4];
      float amax = 0.f;
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          const float gt = acc[i][jj][x];
          h[jj][x] = gt / (1.0f + expf(-gt)) * acc[i][jj + 2][x];
          amax = fmaxf(amax, fabsf(h[jj][x]));
        }
      amax = fmaxf(amax, __shfl_xor(amax, 16));        // the row's 32 hidden values sit in the 4 lanes m16 + 16 g
      amax = fmaxf(amax, __shfl_xor(amax, 32));
      if (gm >= M || tile_n * 32 >= N) continue;
      const int e = mx_block_exponent(amax, 8);
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
        *reinterpret_cast<unsigned*>(codes + (size_t)gm * N + tile_n * 32 + jj * 16 + 4 * g) = mx_pack4_e4m3(h[jj][0], h[jj][1], h[jj][2], h[jj][3], e);
      if (g == 0) {
        out_sc[(size_t)gm * nbp + mx_ascale_index(tile_n)] = (uint8_t)(e + 127);
        if (tile_n == 0) for (int b = N >> 5; b < nbp; ++b) out_sc[(size_t)gm * nbp + mx_ascale_index(b)] = 0;   // scale bytes beyond F
      }
    }
  } else {
    float* cs = (float*)out + (size_t)blockIdx.z * M * N;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int gm = m0 + wv * (MI * 16) + i * 16 + m16;
      if (gm >= M) continue;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int gn = (tile_n * NT + j) * 16 + 4 * g;
        if (gn < N) *reinterpret_cast<f32x4*>(cs + (size_t)gm * N + gn) = acc[i][j];       // N % 16 == 0: whole groups of 4 columns
      }
    }
  }
}

// Row tiles serve the decode-sized row counts below the tiled kernel's.  Tiles are 64 rows high at every row count
// (with the 4-bit weights a tile's traffic is mostly its activation rows, so taking the weights once per 64 rows costs
// little, and three such workgroups fit a compute unit: measured at 192 / 256 rows against 128- and 256-row tiles:
// decode step -5 %); K runs: about 256 workgroups (128, 384, 512: slower), whole groups of 4 chunks.
constexpr int MXR_BM = 64, MXR_STAGES = 4;
static bool gemm_mx_tile_applies(int M, int N, int K);
static bool gemm_mx_rows_applies(int M, int N, int K) {
  return M >= 1 && M <= 1024 && N >= 256 && (N % 16) == 0 && K >= 512 && (K % 128) == 0 && !gemm_mx_tile_applies(M, N, K);
}
static int gemm_mx_rows_slabs(int M, int N, int K) {
  const int tiles = ((N + 63) / 64) * ((M + MXR_BM - 1) / MXR_BM), n_cgrp = ((K >> 7) + 3) >> 2;
  int S = 256 / tiles; if (S < 1) S = 1;
  if (S > n_cgrp) S = n_cgrp;
  const int gpz = (n_cgrp + S - 1) / S;
  return (n_cgrp + gpz - 1) / gpz;              // no empty run
}
template <int EPI>
static void mx_rows_launch(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const uint8_t* w, const uint8_t* w_sc, void* out,
                           uint8_t* out_sc, int M, int N, int K, int col_tiles, int S) {
  constexpr int LDS_BYTES = MXR_STAGES * (MXR_BM * 128 + 4096) + 2 * (4 * 256 + 4 * (MXR_BM / 64) * 256);     // stages + two scale areas
  // opt-in to more than 64 KB of dynamic LDS: once per template instance, thread-safe (initialisation of a local static)
  static const hipError_t attr_once = hipFuncSetAttribute((const void*)k_gemm_mx_rows<EPI, MXR_BM, MXR_STAGES>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  (void)attr_once;
  hipLaunchKernelGGL((k_gemm_mx_rows<EPI, MXR_BM, MXR_STAGES>), dim3(col_tiles, (M + MXR_BM - 1) / MXR_BM, S), dim3(256), LDS_BYTES, s,
                     a, a_sc, w, w_sc, out, out_sc, M, N, K, RopeEpi{});
}

// QKV projection of a decode step with S3 (rotary embedding, gate logit, cache appends) as its epilogue: 64 rows x 128
// columns per workgroup (a wave = 16 rows x one or two whole heads), whole K; no float QKV matrix, no append kernel.
// From 65 rows on (two row tiles: with fewer the whole-K tiles are too few workgroups; measured at batch 64, 2048-token
// context: L = 2 / 3 / 4 step -2 / -1 / -2 %, 64 rows equal, 32 rows and fewer +2-3 %)
bool gemm_mx_rope_rows_applies(int M, int N, int K, int D) {
  return M > 64 && M <= 1024 && (N % 128) == 0 && K >= 128 && (K % 128) == 0 && (D == 64 || D == 128);
}
template <int D, typename KT>
static void mx_rope_launch(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const uint8_t* w, const uint8_t* w_sc, int M, int N, int K,
                           const RopeEpi& ep) {
  constexpr int LDS_BYTES = MXR_STAGES * (MXR_BM * 128 + 8192) + 2 * (8 * 256 + 4 * (MXR_BM / 64) * 256);
  static const hipError_t attr_once = hipFuncSetAttribute((const void*)k_gemm_mx_rows<MXR_ROPE, MXR_BM, MXR_STAGES, 8, D, KT>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  (void)attr_once;
  hipLaunchKernelGGL((k_gemm_mx_rows<MXR_ROPE, MXR_BM, MXR_STAGES, 8, D, KT>), dim3(N / 128, (M + MXR_BM - 1) / MXR_BM, 1), dim3(256), LDS_BYTES, s,
                     a, a_sc, w, w_sc, nullptr, nullptr, M, N, K, ep);
}
void launch_gemm_mx_rope_rows(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const uint8_t* wqkv, const uint8_t* wqkv_sc, int M, int N,
                              int K, const float* gate_w, const float* gate_b, bf16_t* q_out, float* z_out, const KvView& kv,
                              const int32_t* pos, int L, const Dims& dm, const double* inv_freq, int mode, bool kv8) {
  const RopeEpi ep{gate_w, gate_b, inv_freq, q_out, z_out, kv, 0, 0, dm.Hq, dm.Hkv, mode, pos, L};
  if (dm.D == 128) {
    if (kv8) mx_rope_launch<128, fp8_t>(s, a, a_sc, wqkv, wqkv_sc, M, N, K, ep);
    else mx_rope_launch<128, bf16_t>(s, a, a_sc, wqkv, wqkv_sc, M, N, K, ep);
  } else {
    if (kv8) mx_rope_launch<64, fp8_t>(s, a, a_sc, wqkv, wqkv_sc, M, N, K, ep);
    else mx_rope_launch<64, bf16_t>(s, a, a_sc, wqkv, wqkv_sc, M, N, K, ep);
  }
}
static void launch_gemm_mx_rows(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const uint8_t* w, const uint8_t* w_sc, float* c,
                                int M, int N, int K) {
  mx_rows_launch<MXR_F32>(s, a, a_sc, w, w_sc, (void*)c, nullptr, M, N, K, (N + 63) / 64, gemm_mx_rows_slabs(M, N, K));
}

// Gate/up projection of a decode step with SwiGLU and the e4m3 block quantiser as its epilogue: codes[M, F] and their
// scale bytes (the down projection's operand) straight from the product
bool gemm_mx_swiglu_rows_applies(int M, int F, int K) {
  return M >= 1 && M <= 1024 && (F % 32) == 0 && F / 32 >= 128 && K >= 512 && (K % 128) == 0 && !gemm_mx_tile_applies(M, 2 * F, K);
}
void launch_gemm_mx_swiglu_rows(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const uint8_t* wgu, const uint8_t* wgu_sc,
                                uint8_t* codes, uint8_t* scales, int M, int F, int K) {
  mx_rows_launch<MXR_SWIGLU>(s, a, a_sc, wgu, wgu_sc, (void*)codes, scales, M, F, K, F / 32, 1);
}

// rows from which the tiled kernel takes over (its 256 x 256 tiles must fill the chip)
static bool gemm_mx_tile_applies(int M, int N, int K) {
  const long tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
  return M >= 512 && tiles >= 128 && (K % 128) == 0 && (N % 16) == 0;
}

// number of [M, N] float slabs the product leaves: one per K range of the streaming kernel, a single one from the
// tiled kernel
int gemm_mx_splits(int M, int N, int K) {
  if (gemm_mx_tile_applies(M, N, K)) return 1;
  if (gemm_mx_rows_applies(M, N, K)) return gemm_mx_rows_slabs(M, N, K);
  return (K + MX_KR - 1) / MX_KR;
}

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
  if (gemm_mx_rows_applies(M, N, K)) { launch_gemm_mx_rows(s, a, a_sc, w, w_sc, c, M, N, K); return; }
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
