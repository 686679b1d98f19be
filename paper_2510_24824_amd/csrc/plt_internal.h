// Internal declarations shared by the translation units of libplt.so (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/plt.h"

namespace plt {

typedef uint16_t bf16_t;  // storage only; arithmetic is always float

__host__ __device__ inline float bf16_to_f32(bf16_t v) {
  union { uint32_t u; float f; } c; c.u = ((uint32_t)v) << 16; return c.f;
}
// round to nearest, ties to even (inputs are finite in this library)
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
  union { uint32_t u; float f; } c; c.f = f;
  uint32_t lsb = (c.u >> 16) & 1u;
  return (bf16_t)((c.u + 0x7FFFu + lsb) >> 16);
}
// e4m3 cache bytes (OCP e4m3fn): hardware conversions; stores saturate at +-448, nearest even
typedef uint8_t fp8_t;
__device__ inline fp8_t f32_to_e4m3(float f) {
  f = fminf(fmaxf(f, -448.f), 448.f);
  return (fp8_t)(__builtin_amdgcn_cvt_pk_fp8_f32(f, f, 0, false) & 0xff);
}
__device__ inline float e4m3_to_f32(fp8_t v) { return __builtin_amdgcn_cvt_f32_fp8((int)v, 0); }
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
// eight e4m3 bytes (two dwords, memory order) -> eight bf16 values, exact
__device__ inline bf16x8 e4m3x8_to_bf16(unsigned a, unsigned b) {
  const bf16x2 r0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(a, 1.0f, false);
  const bf16x2 r1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(a, 1.0f, true);
  const bf16x2 r2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(b, 1.0f, false);
  const bf16x2 r3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(b, 1.0f, true);
  const bf16x4 lo = __builtin_shufflevector(r0, r1, 0, 1, 2, 3);
  const bf16x4 hi = __builtin_shufflevector(r2, r3, 0, 1, 2, 3);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}
// 16-byte load with the non-temporal hint: for the cache contents that decode attention streams
// once per step, so that they do not push the step's small, re-read buffers (activations, split-K
// slabs) out of the last-level cache (the same hint on the GEMMs' weight stream measured neutral)
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
__device__ inline uint4 ldg16_stream(const void* p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
}
// ---- reductions over lanes on the vector ALU (no trip through the LDS crossbar) ----
// Exchange step S of an all-to-all reduction over the 16 lanes of a row (lanes that share lane / 16): pairs, then
// pairs of pairs, then the two quads of a half row (mirrored: every lane of a quad already holds the quad's
// result), then the two half rows.  After the four steps every lane has combined all 16.
template <int S, typename V>
__device__ inline V row16_xchg(V x) {
  constexpr int ctrl = S == 0 ? 0xB1 : S == 1 ? 0x4E : S == 2 ? 0x141 : 0x140;   // quad_perm 1032, quad_perm 2301, row_half_mirror, row_mirror
  const int u = __builtin_bit_cast(int, x);
  return __builtin_bit_cast(V, __builtin_amdgcn_update_dpp(0, u, ctrl, 0xf, 0xf, true));   // (every lane has a source lane)
}

// The same over the four lanes r, r + 16, r + 32, r + 48 (one lane of each row): gfx950's row swap and half-wave
// swap, which run on the vector ALU; given two copies of one value, combining the two registers after a swap
// combines the pairs.  Written as asm: the compiler folds the builtin's two results into one.  The s_nop cover the
// instructions' read/write hazards.
#define PLT_ROW4_OP(NAME, T, CONSTRAINT, INSTR)                                                                         \
  __device__ __forceinline__ T NAME(T v) {                                                                              \
    T a = v, b = v;                                                                                                     \
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1\n\t" INSTR " %0, %0, %1\n\tv_mov_b32 %1, %0\n\ts_nop 1\n\t" \
                 "v_permlane32_swap_b32 %0, %1\n\ts_nop 1\n\t" INSTR " %0, %0, %1"                                         \
                 : "+" CONSTRAINT(a), "+" CONSTRAINT(b));                                                               \
    return a;                                                                                                           \
  }
PLT_ROW4_OP(row4_max_f32, float, "v", "v_max_f32")
PLT_ROW4_OP(row4_add_f32, float, "v", "v_add_f32")
PLT_ROW4_OP(row4_min_i32, int, "v", "v_min_i32")
#undef PLT_ROW4_OP
__device__ __forceinline__ float wave_max_f32(float v) {
  v = fmaxf(v, row16_xchg<0>(v)); v = fmaxf(v, row16_xchg<1>(v)); v = fmaxf(v, row16_xchg<2>(v)); v = fmaxf(v, row16_xchg<3>(v));
  return row4_max_f32(v);
}
__device__ __forceinline__ float wave_add_f32(float v) {
  v += row16_xchg<0>(v); v += row16_xchg<1>(v); v += row16_xchg<2>(v); v += row16_xchg<3>(v);
  return row4_add_f32(v);
}
__device__ __forceinline__ int wave_min_i32(int v) {
  v = min(v, row16_xchg<0>(v)); v = min(v, row16_xchg<1>(v)); v = min(v, row16_xchg<2>(v)); v = min(v, row16_xchg<3>(v));
  return row4_min_i32(v);
}

template <typename T> __device__ inline float ld(const T* p);
template <> __device__ inline float ld<float>(const float* p) { return *p; }
template <> __device__ inline float ld<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ inline void st(T* p, float v);
template <> __device__ inline void st<float>(float* p, float v) { *p = v; }
template <> __device__ inline void st<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }
template <> __device__ inline float ld<fp8_t>(const fp8_t* p) { return e4m3_to_f32(*p); }
template <> __device__ inline void st<fp8_t>(fp8_t* p, float v) { *p = f32_to_e4m3(v); }

inline int pad32(int n) { return (n + 31) & ~31; }
// cache rows are padded to whole attention tiles: 32 positions, 64 for one-byte (e4m3) caches
inline int pad_kv(int n, bool fp8) { return fp8 ? (n + 63) & ~63 : pad32(n); }

// Index of element (pos, f) inside one K stream.  float caches: row-major [n_pad][D].  bf16 and
// e4m3 caches: tiles of 32 (64) positions stored in the order the decode attention kernel's
// matrix-core loads consume them, [sub-tile a][feature chunk kk][row m][lane group g][16 bytes], where
// lane (m, g) of load (a, kk) holds the 16 bytes of key 8*(m>>2) + (m&3) + 4a, features kk*32 + 8g ..
// (bf16; e4m3: key 16*(m>>2) + (m&3) + 4a, features kk*64 + 16g ..): every wavefront load is then one
// contiguous 1 KB (the lanes read it in a permuted order, which the memory pipeline does not mind), which
// streams measurably faster from HBM than 16 separate 64-byte row pieces, and the four pieces of one key
// (g = 0..3) are 64 adjacent bytes, so appending a key dirties one cache line per feature chunk kk.
template <typename KT> __host__ __device__ inline size_t kblk_index(int pos, int f, int D);
template <> __host__ __device__ inline size_t kblk_index<float>(int pos, int f, int D) { return (size_t)pos * D + f; }
template <> __host__ __device__ inline size_t kblk_index<bf16_t>(int pos, int f, int D) {
  const int t = pos >> 5, j = pos & 31;
  const int a = (j >> 2) & 1, m = ((j >> 3) << 2) | (j & 3);
  const int kk = f >> 5, g = (f >> 3) & 3, e = f & 7;
  return (size_t)t * 32 * D + (size_t)(((a * (D >> 5) + kk) * 64 + m * 4 + g) * 8 + e);
}
template <> __host__ __device__ inline size_t kblk_index<uint8_t>(int pos, int f, int D) {
  const int t = pos >> 6, j = pos & 63;
  const int a = (j >> 2) & 3, m = ((j >> 4) << 2) | (j & 3);
  const int kk = f >> 6, g = (f >> 4) & 3, e = f & 15;
  return (size_t)t * 64 * D + (size_t)(((a * (D >> 6) + kk) * 64 + m * 4 + g) * 16 + e);
}

// Index of element (pos, d) inside one V stream stored as blocks of 32 positions.  float caches: [n_pad/32][D][32],
// position fastest.  bf16 and e4m3 caches: the block is cut into 16-byte chunks of CH = 8 (16) consecutive
// positions of one feature, the unit a matrix-core lane loads, ordered [d / 16][position chunk][d % 16]: the 64
// chunks one wavefront load of the decode attention kernel fetches (16 features x 32 positions) are one contiguous
// KiB, and the chunks that the append of ONE position touches (one per feature) lie 16 in a row, so a new
// position dirties D/8 cache lines of 128 bytes per head instead of the D/2 it would with whole feature rows.
template <typename KT> __host__ __device__ inline size_t vblk_index(int pos, int d, int D);
template <> __host__ __device__ inline size_t vblk_index<float>(int pos, int d, int D) {
  return (size_t)(pos >> 5) * (size_t)(D * 32) + (size_t)d * 32 + (size_t)(pos & 31);
}
template <> __host__ __device__ inline size_t vblk_index<bf16_t>(int pos, int d, int D) {
  const int j = pos & 31;
  return (size_t)(pos >> 5) * (size_t)(D * 32) + (size_t)((((d >> 4) * 4 + (j >> 3)) * 16 + (d & 15)) * 8 + (j & 7));
}
template <> __host__ __device__ inline size_t vblk_index<uint8_t>(int pos, int d, int D) {
  const int j = pos & 31;
  return (size_t)(pos >> 5) * (size_t)(D * 32) + (size_t)((((d >> 4) * 2 + (j >> 4)) * 16 + (d & 15)) * 16 + (j & 15));
}

// How a row of the activation matrices maps to (sequence, position, loop stage).
//  decode : rows_per_seq = L, row = b*L + l, position = pos[b]
//  prefill: rows_per_seq = n, row = b*n + p, loop stage = loop_fixed
struct RowMap {
  int prefill;        // 0 decode, 1 prefill
  int rows_per_seq;   // L (decode) or n (prefill)
  int loop_fixed;     // prefill: 0-based loop stage of every row
  const int32_t* pos; // decode: device array [B] of the position being consumed
};
__device__ inline void row_decode(const RowMap& rm, int r, int& b, int& p, int& l) {
  b = r / rm.rows_per_seq;
  int i = r - b * rm.rows_per_seq;
  if (rm.prefill) { p = i; l = rm.loop_fixed; } else { p = rm.pos[b]; l = i; }
}

// Geometry of one layer's caches as the attention and append kernels see them.
struct KvView {
  void* k_share;   // [B, Hkv, n_pad, D] (float) / tiled, see kblk_index (bf16, e4m3)
  void* v_share;   // [B, Hkv, n_pad/32, D, 32]
  void* k_ring;    // [B, L-1, Hkv, w_pad, D]        (null when L == 1 / vanilla mode)
  void* v_ring;    // [B, L-1, Hkv, w_pad/32, D, 32]
  void* k_loc;     // prefill only: this loop's own K for the chunk [Bc, Hkv, n_pad_loc, D]
  void* v_loc;     // prefill only: [Bc, Hkv, n_pad_loc/32, D, 32]
  int n_pad, w_pad, n_pad_loc;
  int w;           // window
  int n_rings;     // L-1
  int b0;          // prefill: first sequence of the chunk (share/ring are indexed by b0 + b)
  size_t cache_stride;   // elements from this layer's cache c to cache c + 1 (per-loop caches)
};

struct Dims { int B, L, Hq, Hkv, D, d, F, V; };

// ---- launchers (each checks nothing; callers validate shapes) --------------------------
// elem_kernels.hip
template <typename T>
void launch_embed(hipStream_t s, const int32_t* tokens, const T* emb, const float* carry,
                  const float* hprev, float* x, int R, int d, RowMap rm, int n_loops, int add_prev, int vocab);
template <typename T>
void launch_resid_norm(hipStream_t s, float* x, int x_row_stride, int x_row_off,
                       const float* partials, int S, size_t slab, const float* gain, float eps,
                       T* a_out, int R, int d);
// T: type of q_out (the model dtype); KT: element type of the caches (T, or fp8_t)
template <typename T, typename KT>
void launch_rope_append(hipStream_t s, const float* qkv, int S, size_t slab, const float* gate_w,
                        const float* gate_b, T* q_out, float* z_out, KvView kv, RowMap rm, int R,
                        Dims dm, const double* inv_freq /* device [D/2]: theta^(-2j/D) */, int first_loop_only);
template <typename T>
void launch_silu_mul(hipStream_t s, const float* gu, int S, size_t slab, T* act, int R, int F);
void launch_argmax(hipStream_t s, const float* lg, int S, size_t slab, float* logits_out,
                   int32_t* next, int B, int V, float* part_v, int* part_i);
int argmax_scratch_elems(int B);   // elements of part_v and of part_i
void launch_carry_update(hipStream_t s, const float* x, float* carry, int B, int L, int d);
void launch_pos_set(hipStream_t s, int32_t* pos, int B, int value, int increment);
void launch_shift_copy(hipStream_t s, const float* x, float* hprev, size_t n);
// clears nbytes at p (16-byte aligned) with a kernel: unlike a memset node, safe inside a captured HIP graph
void launch_fill_zero(hipStream_t s, void* p, size_t nbytes);
template <typename T>
void launch_pack_k(hipStream_t s, const T* src, T* dst, int S, int n, int n_pad, int D);
template <typename T>
void launch_pack_v(hipStream_t s, const T* src, T* dst, int S, int n, int n_pad, int D);
template <typename T>
void launch_unpack_v(hipStream_t s, const T* src, T* dst, int S, int n, int n_pad, int D);
template <typename T>
void launch_unpack_k(hipStream_t s, const T* src, T* dst, int S, int n, int n_pad, int D);
void launch_prefill_carry(hipStream_t s, const float* x, float* carry, int b0, int Bc, int n,
                          int L, int l, int d);

// gemm_f32.hip / gemm_mfma.hip : c[s][M][N] slabs (float) = a[M,K] * w[N,K]^T
void launch_gemm_f32(hipStream_t s, const float* a, const float* w, float* c, int M, int N, int K);
int gemm_bf16_splits(int M, int N, int K);
void launch_gemm_bf16(hipStream_t s, const bf16_t* a, const bf16_t* w, float* c, int M, int N,
                      int K, int splits);
// gemm_big.hip: many rows (prefill), 256 x 256 tiles, no split-K; optional fused SwiGLU epilogue
bool gemm_big_applies(int M, int N, int K);
void launch_gemm_big(hipStream_t s, const bf16_t* a, const bf16_t* w, float* c, int M, int N, int K);
void launch_gemm_big_resid(hipStream_t s, const bf16_t* a, const bf16_t* w, float* x, int M, int N, int K);   // x += a w^T
void launch_gemm_big_swiglu(hipStream_t s, const bf16_t* a, const bf16_t* wgu, bf16_t* act, int M, int F, int K);
// QKV projection of a prefill chunk (rows = whole sequences of n positions) with the rotary embedding, the gate logit
// and the cache appends as its epilogue; same outputs as launch_gemm_big + launch_rope_append without the float matrix
bool gemm_rope_rows_applies(int M, int N, int K, int D);        // the decode-row form: row (b, l) at position pos[b]
void launch_gemm_rope_rows(hipStream_t s, const bf16_t* a, const bf16_t* wqkv, int M, int N, int K, const float* gate_w,
                           const float* gate_b, bf16_t* q_out, float* z_out, const KvView& kv, const int32_t* pos, int L,
                           const Dims& dm, const double* inv_freq, int mode, bool kv8);
bool gemm_rope_applies(int M, int N, int K, int D);
void launch_gemm_big_rope(hipStream_t s, const bf16_t* a, const bf16_t* wqkv, int M, int N, int K, const float* gate_w,
                          const float* gate_b, bf16_t* q_out, float* z_out, const KvView& kv, int n, int loop, const Dims& dm,
                          const double* inv_freq, int mode, bool kv8);
// decode rows (M <= 256): the gate/up projection with the SwiGLU fused, whole K per workgroup, no slabs
bool gemm_swiglu_rows_applies(int M, int F, int K);
int gemm_rows_split_slabs(int M, int N, int K);
void launch_gemm_rows_split(hipStream_t s, const bf16_t* a, const bf16_t* w, float* c, int M, int N, int K);
void launch_gemm_swiglu_rows(hipStream_t s, const bf16_t* a, const bf16_t* wgu, bf16_t* act, int M, int F, int K);
// picks the weight-streaming kernel for few rows, the big-tile one for many, the small-tile one between
int gemm_bf16_splits_any(int M, int N, int K);
void launch_gemm_bf16_any(hipStream_t s, const bf16_t* a, const bf16_t* w, float* c, int M, int N, int K);

// Expert matrices [N][K] of bf16 models are stored strip by strip (16 rows) in the order the grouped GEMM's
// matrix-core loads consume them: [strip][32-wide k chunk][lane = 16 g + m][8 elements], where lane (m, g)
// holds row 16*strip + m, columns 32*chunk + 8 g ..: one wavefront load is one contiguous KiB and a
// strip is one contiguous stream.  N is a multiple of 16 and K of 32.
__host__ __device__ inline size_t moe_wtile_index(int n, int k, int K) {
  return ((size_t)(n >> 4) * (K >> 5) + (k >> 5)) * 512 + (size_t)((((k >> 3) & 3) * 16 + (n & 15)) * 8 + (k & 7));
}
// ---- microscaling (MX) operands of the low-bit projections: see gemm_mx.hip for the formats
// byte that holds weight element (n, k) of an [N, K] matrix (low nibble: even k): strips of 16 rows, chunks of
// 128 k, inside a chunk lane 16 g + m holds row m, k = 32 g .. 32 g + 31 in 16 bytes
__host__ __device__ inline size_t mx_wcode_index(int n, int k, int K) {
  return ((size_t)(n >> 4) * (K >> 7) + (k >> 7)) * 1024 + (size_t)((((k >> 5) & 3) * 16 + (n & 15)) * 16 + ((k & 31) >> 1));
}
// scale byte of weight row n, k block b (32 k): [strip][group of 4 chunks][lane][chunk in group]
__host__ __device__ inline size_t mx_wscale_index(int n, int b, int K) {
  const int chunk = b >> 2, g = b & 3, n_cgrp = ((K >> 7) + 3) >> 2;
  return (((size_t)(n >> 4) * n_cgrp + (chunk >> 2)) * 64 + g * 16 + (n & 15)) * 4 + (chunk & 3);
}
__host__ __device__ inline size_t mx_wscale_bytes(int N, int K) { return (size_t)(N >> 4) * ((((K >> 7) + 3) >> 2)) * 256; }
// scale byte of k block b inside one activation row: groups of 16 blocks stored [g = b mod 4][c = (b / 4) mod 4]
__host__ __device__ inline int mx_ascale_index(int b) { return (b >> 4) * 16 + (b & 3) * 4 + ((b >> 2) & 3); }
__host__ __device__ inline int mx_ascale_row_bytes(int K) { return ((K + 511) >> 9) * 16; }
// scale exponent of a block with largest magnitude amax: floor(log2(amax)) - emax, clamped; all-zero block: -127
__device__ inline int mx_block_exponent(float amax, int emax) {
  if (!(amax > 0.f)) return -127;
  int e = ilogbf(amax) - emax;
  return e < -127 ? -127 : (e > 127 ? 127 : e);
}
// four consecutive values of a block with exponent e -> four e4m3 bytes (memory order)
__device__ inline unsigned mx_pack4_e4m3(float a, float b, float c, float d, int e) {
  return (unsigned)f32_to_e4m3(ldexpf(a, -e)) | ((unsigned)f32_to_e4m3(ldexpf(b, -e)) << 8) |
         ((unsigned)f32_to_e4m3(ldexpf(c, -e)) << 16) | ((unsigned)f32_to_e4m3(ldexpf(d, -e)) << 24);
}
// elem_kernels.hip: the residual/norm and SwiGLU kernels with the e4m3 block quantiser fused (low-bit models)
bool resid_norm_mx_applies(int d);
void launch_resid_norm_mx(hipStream_t s, float* x, const float* partials, int S, size_t slab, const float* gain, float eps,
                          uint8_t* codes, uint8_t* scales, int R, int d);
void launch_silu_mul_mx(hipStream_t s, const float* gu, int S, size_t slab, uint8_t* codes, uint8_t* scales, int R, int F);
// LDS slice of the low-bit GEMMs: one K range of 1024 per row = 1024 code bytes (+ pad) and 32 scale bytes
constexpr int MX_KR = 1024, MX_LDA = MX_KR + 16, MX_SB = MX_KR / 32;
// gemm_mx.hip
void launch_mx_quant_w(hipStream_t s, const bf16_t* w, uint8_t* codes, uint8_t* scales, int N, int K);
template <typename T>
void launch_mx_quant_a(hipStream_t s, const T* a, uint8_t* codes, uint8_t* scales, int M, int K);
int gemm_mx_splits(int M, int N, int K);
void launch_gemm_mx(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const uint8_t* w, const uint8_t* w_sc, float* c,
                    int M, int N, int K);
// decode rows: QKV projection with S3 (rotary embedding, gate logit, cache appends) as its epilogue
bool gemm_mx_rope_rows_applies(int M, int N, int K, int D);
void launch_gemm_mx_rope_rows(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const uint8_t* wqkv, const uint8_t* wqkv_sc, int M, int N,
                              int K, const float* gate_w, const float* gate_b, bf16_t* q_out, float* z_out, const KvView& kv,
                              const int32_t* pos, int L, const Dims& dm, const double* inv_freq, int mode, bool kv8);
// decode rows: gate/up projection with SwiGLU and the e4m3 block quantiser as its epilogue (codes[M, F] + scale bytes)
bool gemm_mx_swiglu_rows_applies(int M, int F, int K);
void launch_gemm_mx_swiglu_rows(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const uint8_t* wgu, const uint8_t* wgu_sc,
                                uint8_t* codes, uint8_t* scales, int M, int F, int K);

// moe.hip : mixture-of-experts feed-forward.  Index arrays of one call (device): the selected experts and
// their probabilities per row, the (row, slot) pairs sorted by expert and every expert's span in that list.
struct MoeIndex { int32_t* sel_e; float* sel_p; int32_t* pair; int32_t* off; int32_t* span /* sort scratch */; };
size_t moe_index_bytes(int R, int k, int E);
MoeIndex moe_index_carve(void* base, int R, int k, int E);
// a [R, d] normed rows; router [E, d]; wgu [E, 2F, d] (per expert: gate rows, then up rows); wdown [E, d, F]
// (bf16: every expert matrix in the strip order of moe_wtile_index; float: row-major);
// act: scratch [R*k, F]; y: k slabs [k][R][d] (slab s, row r = p * the output of row r's s-th expert)
template <typename T>
void launch_moe_ffn(hipStream_t s, const T* a, const T* router, const T* wgu, const T* wdown, T* act, float* y,
                    MoeIndex mi, int R, int d, int F, int E, int k);
// the same layer on low-bit operands: a as e4m3 codes + block scales [R, d]; router bf16 [E, d]; per expert the
// gate/up matrix [2F, d] and the down matrix [d, F] as e2m1 codes + scales in the layouts of gemm_mx.hip
// (expert e's tensors start at e times the size of one); act_codes / act_scales: scratch [R*k, F] e4m3 blocks
// (the pad bytes of act_scales must be zero)
void launch_moe_ffn_mx(hipStream_t s, const uint8_t* a, const uint8_t* a_sc, const bf16_t* router, const uint8_t* wgu,
                       const uint8_t* wgu_sc, const uint8_t* wdown, const uint8_t* wdown_sc, uint8_t* act_codes,
                       uint8_t* act_scales, float* y, MoeIndex mi, int R, int d, int F, int E, int k);

// attn_f32.hip : one wave per (row, query head), float storage
void launch_attn_f32(hipStream_t s, const float* q, const float* z, float* y, KvView kv,
                     RowMap rm, int R, Dims dm, int plain);

// attn_mfma.hip : bf16 q / y, caches in bf16 or e4m3 (kv_fp8), MFMA tiles
size_t attn_mfma_scratch_bytes(int B, int L, int Hq, int Hkv, int D, int max_splits = 64);
int attn_mfma_max_default_splits(int B, int Hkv);
int attn_mfma_default_splits(int B, int Hkv, int L, int G, int n_ctx, int kv_fp8 = 0);
void launch_attn_decode_mfma(hipStream_t s, const bf16_t* q, const float* z, bf16_t* y, KvView kv,
                             const int32_t* pos, int n_ctx_uniform, int n_ring_uniform,
                             Dims dm, int plain, void* scratch, int n_splits,
                             int l_off = 0, int l_stride = 0 /* rows per sequence in q / y; 0 = dm.L */,
                             int kv_fp8 = 0, int scratch_splits = 64 /* max_splits the scratch was sized with */,
                             uint8_t* y_codes = nullptr, uint8_t* y_scales = nullptr /* low-bit models: y as e4m3
                             blocks [rows, Hq*D] + scale bytes instead of bf16 (Hq*D a multiple of 512) */);
// local_tmp: float scratch [Bc*n, Hq*D] (used by loops >= 2 only)
void launch_attn_prefill_mfma(hipStream_t s, const bf16_t* q, const float* z, bf16_t* y, float* local_tmp,
                              KvView kv, int Bc, int n, int loop, Dims dm, int plain, int kv_fp8 = 0);

}  // namespace plt
