// Fused PLT attention on gfx950 matrix cores, bf16 storage, float statistics.
//
// What it computes, for the (up to 16) query rows that share one K/V stream:
//   first-loop rows : y = Attn(q, K_share, V_share)                                  [Sec. 2.2.1]
//   other rows      : y = g * SWA(q, own K/V, w) + (1 - g) * Attn(q, K_share, V_share),
//                     g = sigmoid(z)                                      [Alg. 3 l.2-5, Eq. (2)]
// The rows are the L loop stages x G query heads of one (sequence, kv head); K_share / V_share are
// streamed from HBM exactly once for all of them.  (The prefill counterpart lives in attn_prefill.hip.)
//
// Tile algebra (one wave, 32 keys at a time, v_mfma_f32_16x16x32_bf16):
//   S^T[key][row] = K[key][:] . Q[row][:]      A = K straight from HBM (16 B per lane; the cache keeps
//                                              K tiles in exactly this load order), B = Q in registers
//   O^T[d][row]  += V^T[d][key] * P^T[key][row]  A = V^T, 16 B per lane thanks to the cache's
//                                              V layout (16-byte chunks of consecutive positions)
// With this orientation a lane owns one query row in S^T, P^T and O^T alike, so the online
// softmax needs no data movement between the two contractions; the row maximum is completed
// with a row swap and a half-wave swap (lanes r, r+16, r+32, r+48).  The four waves of a workgroup take
// alternate tiles and merge their (m, l, O) states through LDS; workgroups that split one
// stream leave (m, l, O) records in an HBM scratch that a small second kernel merges (a
// device-scope fence per workgroup costs far more on this multi-die part than a launch).
//
// e4m3 caches (F8 = true): the same algebra on tiles of 64 keys.  A lane still fetches 16 bytes
// per load, now 16 features of a key row (two MFMA K-chunks; the query fragments are laid out to
// match) or 16 positions of a V row; v_cvt_scalef32_pk_bf16_fp8 expands the bytes exactly to the
// bf16 operands the matrix cores take, so only the bytes streamed from HBM change (halved).
#include "plt_internal.h"

namespace plt {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) float f32x8;

#define NEG_INF (-INFINITY)

__device__ inline bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ inline uint4 ldg16(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }

template <int D>
struct WaveState {
  float m;                 // running row maximum (log2 domain), identical in the 4 lanes of a row
  float l;                 // this lane's share of the row's softmax denominator
  f32x4 acc[D / 16];       // O^T[d = 16*dt + 4*g + i][row]
  __device__ void init() {
    m = NEG_INF; l = 0.f;
#pragma unroll
    for (int i = 0; i < D / 16; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
};

template <int D, bool F8> struct KvTile;
template <int D>
struct KvTile<D, false> {  // 32 keys of bf16
  uint4 k[2][D / 32];      // two 16-key sub-tiles, D/32 chunks of 8 features each
  uint4 v[D / 16];         // D/16 groups of 16 features, 8 keys per lane
};
template <int D>
struct KvTile<D, true> {   // 64 keys of e4m3
  uint4 k[4][D / 64];      // four 16-key sub-tiles, D/64 chunks of 16 features each
  uint4 v[D / 16];         // D/16 groups of 16 features, 16 keys per lane
};

// kt -> the tile's K block (32 keys, stored in load order: see kblk_index); vt -> the tile's V block (vblk_index)
template <int D>
__device__ inline void load_tile_k(KvTile<D, false>& t, const char* __restrict__ kt, int m16, int g) {
  const char* kp = kt + (m16 * 4 + g) * 16;      // A-row m16 of sub-tile a <-> key 8*(m16>>2) + (m16&3) + 4a
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk)
      t.k[a][kk] = ldg16_stream(kp + (a * (D / 32) + kk) * 1024);
}
template <int D>
__device__ inline void load_tile_v(KvTile<D, false>& t, const char* __restrict__ vt, int m16, int g) {
  const char* vp = vt + (g * 16 + m16) * 16;      // chunk (dt, g, m16): positions 8g .. 8g+7 of feature 16 dt + m16
#pragma unroll
  for (int dt = 0; dt < D / 16; ++dt) t.v[dt] = ldg16_stream(vp + dt * 1024);
}
// e4m3: kt -> the tile's K block (64 keys, load order); vt -> the tile's two V blocks
template <int D>
__device__ inline void load_tile_k(KvTile<D, true>& t, const char* __restrict__ kt, int m16, int g) {
  const char* kp = kt + (m16 * 4 + g) * 16;      // A-row m16 of sub-tile a <-> key 16*(m16>>2) + (m16&3) + 4a
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int kk = 0; kk < D / 64; ++kk)
      t.k[a][kk] = ldg16_stream(kp + (a * (D / 64) + kk) * 1024);
}
template <int D>
__device__ inline void load_tile_v(KvTile<D, true>& t, const char* __restrict__ vt, int m16, int g) {
  // lane g: positions 16g .. 16g+15 of the tile = chunk (dt, g & 1, m16) of block g / 2
  const char* vb = vt + (size_t)(g >> 1) * (D * 32) + ((g & 1) * 16 + m16) * 16;
#pragma unroll
  for (int dt = 0; dt < D / 16; ++dt) t.v[dt] = ldg16_stream(vb + dt * 512);
}

// One 32-key step of the online softmax.  valid(j) tells whether key j (0..7 -> tile key 8g+j)
// may be attended by this lane's row; it is consulted only when need_mask is set.
// mid() runs between the two contractions, when the K half of the tile is no longer needed, and end()
// after the second one, when the V half is not either: the caller refills those registers there.
template <int D, typename Valid, typename Mid, typename End>
__device__ inline void tile_step(WaveState<D>& st, KvTile<D, false>& t, const uint4 (&qf)[D / 32],
                                 float scale_log2, bool need_mask, Valid valid, Mid mid, End end) {
  f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kk = 0; kk < D / 32; ++kk) {
    s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(t.k[0][kk]), as_bf16x8(qf[kk]), s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(t.k[1][kk]), as_bf16x8(qf[kk]), s1, 0, 0, 0);
  }
  mid();
  float sv[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) { sv[i] = s0[i]; sv[4 + i] = s1[i]; }
  if (need_mask) {
#pragma unroll
    for (int j = 0; j < 8; ++j) if (!valid(j)) sv[j] = NEG_INF;
  }
  float mx = sv[0];
#pragma unroll
  for (int j = 1; j < 8; ++j) mx = fmaxf(mx, sv[j]);
  mx = row4_max_f32(mx);
  const float m_new = fmaxf(st.m, mx * scale_log2);      // the scale is positive: max and scaling commute
  const float m_safe = (m_new == NEG_INF) ? 0.f : m_new;
  const float alpha = __builtin_amdgcn_exp2f(st.m - m_safe);
  f32x8 p;
  float ps = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) { p[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[j], scale_log2, -m_safe)); ps += p[j]; }
  st.l = st.l * alpha + ps;
  st.m = m_new;
  const bf16x8 pb = __builtin_convertvector(p, bf16x8);
  // alpha == 1 in every lane (no row raised its maximum: the usual case after the first few tiles): the rescale
  // of the accumulators is skipped for the whole wave
  if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) { st.acc[dt][0] *= alpha; st.acc[dt][1] *= alpha; st.acc[dt][2] *= alpha; st.acc[dt][3] *= alpha; }
  }
#pragma unroll
  for (int dt = 0; dt < D / 16; ++dt)
    st.acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(t.v[dt]), pb, st.acc[dt], 0, 0, 0);
  end();
}

// The same step on a 64-key e4m3 tile.  valid(j), j = 0..15 <-> tile key 16g + j.  qf[2c + h] holds
// the lane's query features c*64 + 16g + 8h .. +7, matching the two halves of a 16-byte key load.
template <int D, typename Valid, typename Mid, typename End>
__device__ inline void tile_step(WaveState<D>& st, KvTile<D, true>& t, const uint4 (&qf)[D / 32],
                                 float scale_log2, bool need_mask, Valid valid, Mid mid, End end) {
  f32x4 s[4];
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    s[a] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < D / 64; ++kk) {
      const uint4 r = t.k[a][kk];
      s[a] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(e4m3x8_to_bf16(r.x, r.y), as_bf16x8(qf[2 * kk]), s[a], 0, 0, 0);
      s[a] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(e4m3x8_to_bf16(r.z, r.w), as_bf16x8(qf[2 * kk + 1]), s[a], 0, 0, 0);
    }
  }
  mid();
  float sv[16];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int i = 0; i < 4; ++i) sv[4 * a + i] = s[a][i];
  if (need_mask) {
#pragma unroll
    for (int j = 0; j < 16; ++j) if (!valid(j)) sv[j] = NEG_INF;
  }
  float mx = sv[0];
#pragma unroll
  for (int j = 1; j < 16; ++j) mx = fmaxf(mx, sv[j]);
  mx = row4_max_f32(mx);
  const float m_new = fmaxf(st.m, mx * scale_log2);      // the scale is positive: max and scaling commute
  const float m_safe = (m_new == NEG_INF) ? 0.f : m_new;
  const float alpha = __builtin_amdgcn_exp2f(st.m - m_safe);
  f32x8 p0, p1;
  float ps = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    p0[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[j], scale_log2, -m_safe));
    p1[j] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[8 + j], scale_log2, -m_safe));
    ps += p0[j] + p1[j];
  }
  st.l = st.l * alpha + ps;
  st.m = m_new;
  const bf16x8 pb0 = __builtin_convertvector(p0, bf16x8), pb1 = __builtin_convertvector(p1, bf16x8);
  if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {      // (as above)
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) { st.acc[dt][0] *= alpha; st.acc[dt][1] *= alpha; st.acc[dt][2] *= alpha; st.acc[dt][3] *= alpha; }
  }
#pragma unroll
  for (int dt = 0; dt < D / 16; ++dt) {
    f32x4 a = st.acc[dt];
    const uint4 r = t.v[dt];
    a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(e4m3x8_to_bf16(r.x, r.y), pb0, a, 0, 0, 0);
    st.acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(e4m3x8_to_bf16(r.z, r.w), pb1, a, 0, 0, 0);
  }
  end();
}

// LDS block used to merge the four waves of a workgroup.
template <int D>
struct WgMerge {
  float m[4][16];
  float l[4][16];
  float acc[4][16][D + 4];
};

// wg_park: a wave leaves its (m, l, O) state in its own part of the LDS block (no barrier inside).
template <int D>
__device__ inline void wg_park(WgMerge<D>& sm, const WaveState<D>& st, int wv, int m16, int g) {
  float l = st.l;
  l = row4_add_f32(l);
  if (g == 0) { sm.m[wv][m16] = st.m; sm.l[wv][m16] = l; }
#pragma unroll
  for (int dt = 0; dt < D / 16; ++dt)
#pragma unroll
    for (int i = 0; i < 4; ++i) sm.acc[wv][m16][dt * 16 + 4 * g + i] = st.acc[dt][i];
}
// wg_collect (after a barrier that follows the four parks): thread tid gets, for row tid/16 and
// features (tid%16)*(D/16) .. +D/16-1, the workgroup-wide unnormalised output o[], the row maximum
// M and the denominator Lsum.
template <int D>
__device__ inline void wg_collect(const WgMerge<D>& sm, float& M, float& Lsum, float (&o)[D / 16]) {
  const int row = threadIdx.x >> 4, dc = (threadIdx.x & 15) * (D / 16);
  M = fmaxf(fmaxf(sm.m[0][row], sm.m[1][row]), fmaxf(sm.m[2][row], sm.m[3][row]));
  Lsum = 0.f;
#pragma unroll
  for (int i = 0; i < D / 16; ++i) o[i] = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float mw = sm.m[w][row];
    const float f = (mw == NEG_INF) ? 0.f : __builtin_amdgcn_exp2f(mw - M);
    Lsum += f * sm.l[w][row];
#pragma unroll
    for (int i = 0; i < D / 16; ++i) o[i] += f * sm.acc[w][row][dc + i];
  }
}
template <int D>
__device__ inline void wg_merge(WgMerge<D>& sm, WaveState<D>& st, int wv, int m16, int g,
                                float& M, float& Lsum, float (&o)[D / 16]) {
  __syncthreads();                       // previous users of sm are done
  wg_park<D>(sm, st, wv, m16, g);
  __syncthreads();
  wg_collect<D>(sm, M, Lsum, o);
}

template <int D>
__device__ inline void store_row(bf16_t* __restrict__ dst, const float (&v)[D / 16]) {
  // D/16 consecutive bf16 values: 4 (D = 64) or 8 (D = 128)
#pragma unroll
  for (int i = 0; i < D / 16; ++i) dst[i] = f32_to_bf16(v[i]);
}

// ------------------------------------------------------------------------------- decode

struct AttnDecArgs {
  const bf16_t* q; const float* z; bf16_t* y;
  const char* k_share; const char* v_share; const char* k_ring; const char* v_ring;   // bf16 or e4m3 elements
  const int32_t* pos;          // per-sequence position being consumed, or null
  int n_ctx_uniform, n_ring_uniform;
  int n_pad, w_pad, w, n_rings;
  int L, Hq, Hkv, G, n_rows, n_rt, n_splits, plain;
  int l_off, l_stride;         // q / y row of (sequence b, loop l) = b * l_stride + l_off + l
  float scale_log2;
  float* part;                 // [stream][rt][split] records of (16 + 16 + 16*D) floats
  float* part_loc;             // [stream][rt] records of 16*D floats (normalised local branch)
  // low-bit models: y leaves as e4m3 blocks of 32 (the input format of the output projection) instead of bf16
  uint8_t* y_codes; uint8_t* y_scales; int y_nbp;   // codes [rows, Hq*D], scale bytes [rows, y_nbp]; null = bf16 y
};

// Normalises the two branches of one row chunk, applies the gate of Eq. (2) and stores y.
// Thread tid covers row tid/16 of row tile rt and features (tid%16)*(D/16) .. +D/16-1.
template <int D>
__device__ inline void finalize_row(const AttnDecArgs& A, int b, int kvh, int rt, int tid, float Lg,
                                    const float (&og)[D / 16], float Ll, const float (&ol)[D / 16]) {
  const int row = rt * 16 + (tid >> 4), dc = (tid & 15) * (D / 16);
  if (row >= A.n_rows) return;
  const int r_loop = row / A.G, r_head = kvh * A.G + row % A.G;
  const bool gated = !A.plain && r_loop > 0;
  float out[D / 16];
  const float invg = Lg > 0.f ? 1.0f / Lg : 0.f;
  if (gated) {
    const float zz = A.z[((size_t)b * (A.L - 1) + (r_loop - 1)) * A.Hq + r_head];
    const float gate = 1.0f / (1.0f + __expf(-zz));
    const float invl = Ll > 0.f ? 1.0f / Ll : 0.f;
#pragma unroll
    for (int i = 0; i < D / 16; ++i) out[i] = gate * (ol[i] * invl) + (1.0f - gate) * (og[i] * invg);
  } else {
#pragma unroll
    for (int i = 0; i < D / 16; ++i) out[i] = og[i] * invg;
  }
  const size_t yrow = (size_t)b * A.l_stride + A.l_off + r_loop;
  if (A.y_codes == nullptr) {
    store_row<D>(A.y + (yrow * A.Hq + r_head) * D + dc, out);
    return;
  }
  // a block of 32 features = 32 / (D/16) consecutive threads of this row (4 for D = 128, 8 for D = 64)
  float amax = 0.f;
#pragma unroll
  for (int i = 0; i < D / 16; ++i) amax = fmaxf(amax, fabsf(out[i]));
  amax = fmaxf(amax, row16_xchg<0>(amax)); amax = fmaxf(amax, row16_xchg<1>(amax));
  if (D == 64) amax = fmaxf(amax, row16_xchg<2>(amax));
  const int e = mx_block_exponent(amax, 8);
  const int col = r_head * D + dc;
  unsigned* dst = reinterpret_cast<unsigned*>(A.y_codes + yrow * (size_t)(A.Hq * D) + col);
#pragma unroll
  for (int i = 0; i < D / 64; ++i) dst[i] = mx_pack4_e4m3(out[4 * i], out[4 * i + 1], out[4 * i + 2], out[4 * i + 3], e);
  if ((col & 31) == 0) A.y_scales[yrow * A.y_nbp + mx_ascale_index(col >> 5)] = (uint8_t)(e + 127);
}

template <int D, bool F8>
__global__ __launch_bounds__(256, 2) void k_attn_decode(AttnDecArgs A) {
  constexpr int TK = F8 ? 64 : 32;            // keys per tile
  constexpr int ES = F8 ? 1 : 2;              // bytes per cache element
  constexpr int KL = F8 ? 16 : 8;             // tile keys per lane group g: TK/4 consecutive ones
  __shared__ WgMerge<D> sm;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, m16 = lane & 15, g = lane >> 4;
  const int split = blockIdx.x % A.n_splits, rt = blockIdx.x / A.n_splits;
  const int kvh = blockIdx.y, b = blockIdx.z;
  const int n_ctx = A.pos ? A.pos[b] + 1 : A.n_ctx_uniform;
  const int n_ring = A.pos ? (A.pos[b] + 1 < A.w ? A.pos[b] + 1 : A.w) : A.n_ring_uniform;
  const size_t stream = (size_t)b * A.Hkv + kvh;

  // this lane's query row (B operand: lane (row, g) holds features kk*32 + g*8 .. +7; for e4m3
  // caches fragment 2c + h holds features c*64 + 16g + 8h .. +7)
  const int qrow = rt * 16 + m16;
  const bool qrow_ok = qrow < A.n_rows;
  const int q_loop = qrow_ok ? qrow / A.G : 0;
  const int q_head = kvh * A.G + (qrow_ok ? qrow % A.G : 0);
  uint4 qf[D / 32];
#pragma unroll
  for (int kk = 0; kk < D / 32; ++kk) {
    qf[kk] = make_uint4(0, 0, 0, 0);
    const int qo = F8 ? (kk >> 1) * 64 + g * 16 + (kk & 1) * 8 : kk * 32 + g * 8;
    if (qrow_ok) qf[kk] = ldg16(A.q + (((size_t)b * A.l_stride + A.l_off + q_loop) * A.Hq + q_head) * D + qo);
  }

  // ---- global branch: this split's share of the shared cache, alternate tiles per wave ----
  const int n_tiles = (n_ctx + TK - 1) / TK;
  const int tps = (n_tiles + A.n_splits - 1) / A.n_splits;
  const int t_beg = split * tps;
  const int t_end = (t_beg + tps < n_tiles) ? t_beg + tps : n_tiles;
  const char* kbase = A.k_share + stream * (size_t)A.n_pad * D * ES;
  const char* vbase = A.v_share + stream * (size_t)A.n_pad * D * ES;
  // ---- local branch (last split only): the valid tiles of the rings of loops 2..L ----
  const bool do_local = !A.plain && A.n_rings > 0 && split == A.n_splits - 1;
  const int tv = (n_ring + TK - 1) / TK;                   // valid tiles per ring
  const int n_loc = do_local ? A.n_rings * tv : 0;
  // One software pipeline over both kinds of tile; wave wv takes entries wv, wv+4, ...  While an
  // entry is being multiplied the next one (of either kind) is already in flight, so the window
  // branch adds no exposed memory latency.  bf16 caches: entries 0..n_my-1 are this split's shared
  // tiles, then the ring tiles, and the two branches keep separate online-softmax states.  e4m3
  // caches (RING_FIRST; their 64-key tiles leave no room for a second state): the ring tiles come
  // first, and when a wave moves on to its shared tiles it parks the window state in LDS and
  // starts over.
  constexpr bool RING_FIRST = F8;
  WaveState<D> st, sl; st.init(); sl.init();
  {
    // Shared tiles are visited in a rotated order that differs from stream to stream (softmax does
    // not care about order): workgroups that run in lockstep then touch different HBM channels
    // instead of the same offset of their equally aligned streams.
    KvTile<D, F8> cur, nxt;
    const int n_my = t_end > t_beg ? t_end - t_beg : 0;    // a late split may own no shared tile
    const int n_ent = n_my + n_loc;
    const int rot = n_my > 0 ? (int)((stream * 13u + (unsigned)split * 7u) % (unsigned)n_my) : 0;
    auto tile_of = [&](int u) { int t = u + rot; if (t >= n_my) t -= n_my; return t_beg + t; };
    auto is_ring = [&](int e) { return RING_FIRST ? e < n_loc : e >= n_my; };
    auto ring_idx = [&](int e) { return RING_FIRST ? e : e - n_my; };
    auto share_idx = [&](int e) { return RING_FIRST ? e - n_loc : e; };
    // which = 1: the K half of entry e, 2: the V half, 3: both
    auto load_entry = [&](KvTile<D, F8>& tl, int e, int which) {
      const char* kp; const char* vp;
      if (!is_ring(e)) {
        const size_t to = (size_t)tile_of(share_idx(e)) * TK * D * ES;
        kp = kbase + to; vp = vbase + to;
      } else {
        const int j = ring_idx(e), rl = j / tv, tr = j - rl * tv;
        const size_t ro = ((((size_t)b * A.n_rings + rl) * A.Hkv + kvh) * (size_t)A.w_pad + (size_t)tr * TK) * D * ES;
        kp = A.k_ring + ro; vp = A.v_ring + ro;
      }
      if (which & 1) load_tile_k<D>(tl, kp, m16, g);
      if (which & 2) load_tile_v<D>(tl, vp, m16, g);
    };
    // Two tile buffers per wave, refilled in halves as soon as a half has been consumed: while entry e
    // is being multiplied, entry e + 4 is resident or in flight, and the K half (then the V half) of
    // entry e + 8 is requested into the registers entry e has just released.  Between one and two
    // tiles per wave are in flight at any time, in the registers of two.
    bool parked = !(RING_FIRST && do_local);     // is the window state already out of the way?
    auto process = [&](KvTile<D, F8>& tl, int e) {
      const int e2 = e + 8;
      auto mid = [&]() { if (e2 < n_ent) load_entry(tl, e2, 1); };
      auto end = [&]() { if (e2 < n_ent) load_entry(tl, e2, 2); };
      if (!is_ring(e)) {
        if (!parked) { wg_park<D>(sm, st, wv, m16, g); st.init(); parked = true; }
        const int t = tile_of(share_idx(e)), kb = t * TK + KL * g;
        tile_step<D>(st, tl, qf, A.scale_log2, (t + 1) * TK > n_ctx, [&](int j) { return kb + j < n_ctx; }, mid, end);
      } else {
        const int j0 = ring_idx(e), rl = j0 / tv, tr = j0 - rl * tv, sb = tr * TK + KL * g;
        const bool mine = qrow_ok && (q_loop == rl + 1);
        tile_step<D>(RING_FIRST ? st : sl, tl, qf, A.scale_log2, true, [&](int j) { return mine && (sb + j < n_ring); }, mid, end);
      }
    };
    KvTile<D, F8>& ta = cur; KvTile<D, F8>& tb = nxt;
    int e = wv;
    if (e < n_ent) load_entry(ta, e, 3);
    if (e + 4 < n_ent) load_entry(tb, e + 4, 3);
    for (; e < n_ent; e += 8) {
      process(ta, e);
      if (e + 4 < n_ent) process(tb, e + 4);
    }
    if (!parked) { wg_park<D>(sm, st, wv, m16, g); st.init(); }   // this wave had ring tiles only
  }
  float Mg, Lg, og[D / 16];
  float Ml = NEG_INF, Ll = 0.f, ol[D / 16];
#pragma unroll
  for (int i = 0; i < D / 16; ++i) ol[i] = 0.f;
  if (RING_FIRST) {
    if (do_local) { __syncthreads(); wg_collect<D>(sm, Ml, Ll, ol); }
    wg_merge<D>(sm, st, wv, m16, g, Mg, Lg, og);
  } else {
    wg_merge<D>(sm, st, wv, m16, g, Mg, Lg, og);
    if (do_local) wg_merge<D>(sm, sl, wv, m16, g, Ml, Ll, ol);
  }

  // ---- thread (row, feature chunk) view from here on ----
  const int dc = (tid & 15) * (D / 16);
  const size_t slot = stream * A.n_rt + rt;
  if (A.n_splits > 1) {
    // several workgroups share this stream: leave (m, l, O) records; k_attn_combine finishes
    const size_t rec = (size_t)(16 + 16 + 16 * D);
    float* pr = A.part + (slot * A.n_splits + split) * rec;
    if ((tid & 15) == 0) { pr[tid >> 4] = Mg; pr[16 + (tid >> 4)] = Lg; }
#pragma unroll
    for (int i = 0; i < D / 16; ++i) pr[32 + (tid >> 4) * D + dc + i] = og[i];
    if (do_local) {
      float* pl = A.part_loc + slot * (size_t)(16 * D);
      const float inv = Ll > 0.f ? 1.0f / Ll : 0.f;
#pragma unroll
      for (int i = 0; i < D / 16; ++i) pl[(tid >> 4) * D + dc + i] = ol[i] * inv;
    }
    return;
  }
  finalize_row<D>(A, b, kvh, rt, tid, Lg, og, Ll, ol);
}

// Merges the split records of one (stream, row tile) in a fixed order (bit-reproducible) and
// applies Eq. (2).  One workgroup per (row tile, kv head, sequence); launched after k_attn_decode
// on the same stream whenever n_splits > 1.
template <int D>
__global__ __launch_bounds__(256) void k_attn_combine(AttnDecArgs A) {
  const int tid = threadIdx.x, rt = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int dc = (tid & 15) * (D / 16);
  const size_t stream = (size_t)b * A.Hkv + kvh, slot = stream * A.n_rt + rt;
  const size_t rec = (size_t)(16 + 16 + 16 * D);
  const float* p0 = A.part + slot * A.n_splits * rec;
  float M = NEG_INF;
  for (int s = 0; s < A.n_splits; ++s) M = fmaxf(M, p0[s * rec + (tid >> 4)]);
  float Lg = 0.f, og[D / 16], Ll = 0.f, ol[D / 16];
#pragma unroll
  for (int i = 0; i < D / 16; ++i) { og[i] = 0.f; ol[i] = 0.f; }
  for (int s = 0; s < A.n_splits; ++s) {
    const float* ps = p0 + s * rec;
    const float ms = ps[tid >> 4];
    const float f = (ms == NEG_INF) ? 0.f : __builtin_amdgcn_exp2f(ms - M);
    Lg += f * ps[16 + (tid >> 4)];
#pragma unroll
    for (int i = 0; i < D / 16; ++i) og[i] += f * ps[32 + (tid >> 4) * D + dc + i];
  }
  if (!A.plain && A.n_rings > 0) {
    const float* pl = A.part_loc + slot * (size_t)(16 * D);
#pragma unroll
    for (int i = 0; i < D / 16; ++i) ol[i] = pl[(tid >> 4) * D + dc + i];
    Ll = 1.f;
  }
  finalize_row<D>(A, b, kvh, rt, tid, Lg, og, Ll, ol);
}

size_t attn_mfma_scratch_bytes(int B, int L, int Hq, int Hkv, int D, int max_splits_in) {
  const int G = Hq / Hkv, n_rt = (L * G + 15) / 16;
  const size_t slots = (size_t)B * Hkv * n_rt;
  const size_t rec = (size_t)(32 + 16 * D) * sizeof(float);
  const size_t max_splits = max_splits_in < 1 ? 1 : (max_splits_in > 64 ? 64 : max_splits_in);
  size_t bytes = slots * max_splits * rec;            // split records
  bytes += slots * (size_t)(16 * D) * sizeof(float);  // local-branch records
  return bytes;
}

// the largest value attn_mfma_default_splits can return for any context length and any rows per stream
int attn_mfma_max_default_splits(int B, int Hkv) {
  const long streams = (long)B * Hkv;
  if (streams >= 256) return 1;
  const int s = (int)((256 + streams - 1) / streams);
  return s > 64 ? 64 : s;
}

int attn_mfma_default_splits(int B, int Hkv, int L, int G, int n_ctx, int kv_fp8) {
  const int n_rt = (L * G + 15) / 16;
  const long streams = (long)B * Hkv * n_rt;
  const int tk = kv_fp8 ? 64 : 32;
  const int n_tiles = (n_ctx + tk - 1) / tk;
  // one workgroup per stream when that already covers every compute unit; else split so that
  // about one workgroup per compute unit exists (more splits only add merge work: measured),
  // keeping >= 8 tiles (2 per wave) per workgroup (an eight-wave workgroup variant measured slower)
  if (streams >= 256) return 1;
  int s = (int)((256 + streams - 1) / streams);
  int cap = n_tiles / 8; if (cap < 1) cap = 1;           // at least two tiles per wave
  if (s > cap) s = cap;
  if (s > 64) s = 64;
  if (s < 1) s = 1;
  return s;
}

void launch_attn_decode_mfma(hipStream_t s, const bf16_t* q, const float* z, bf16_t* y, KvView kv,
                             const int32_t* pos, int n_ctx_uniform, int n_ring_uniform, Dims dm,
                             int plain, void* scratch, int n_splits, int l_off, int l_stride, int kv_fp8,
                             int scratch_splits, uint8_t* y_codes, uint8_t* y_scales) {
  AttnDecArgs A;
  A.y_codes = y_codes; A.y_scales = y_scales; A.y_nbp = mx_ascale_row_bytes(dm.Hq * dm.D);
  A.l_off = l_off; A.l_stride = l_stride > 0 ? l_stride : dm.L;
  A.q = q; A.z = z; A.y = y;
  A.k_share = (const char*)kv.k_share; A.v_share = (const char*)kv.v_share;
  A.k_ring = (const char*)kv.k_ring; A.v_ring = (const char*)kv.v_ring;
  A.pos = pos; A.n_ctx_uniform = n_ctx_uniform; A.n_ring_uniform = n_ring_uniform;
  A.n_pad = kv.n_pad; A.w_pad = kv.w_pad; A.w = kv.w; A.n_rings = plain ? 0 : kv.n_rings;
  A.L = dm.L; A.Hq = dm.Hq; A.Hkv = dm.Hkv; A.G = dm.Hq / dm.Hkv;
  A.n_rows = dm.L * A.G; A.n_rt = (A.n_rows + 15) / 16;
  if (scratch_splits < 1 || scratch_splits > 64) scratch_splits = 64;    // split records the scratch was sized for
  A.n_splits = n_splits < 1 ? 1 : (n_splits > scratch_splits ? scratch_splits : n_splits);
  A.plain = plain;
  A.scale_log2 = 1.4426950408889634f / sqrtf((float)dm.D);
  const size_t slots = (size_t)dm.B * dm.Hkv * A.n_rt;
  const size_t rec = (size_t)(32 + 16 * dm.D);
  A.part = (float*)scratch;
  A.part_loc = A.part + slots * (size_t)scratch_splits * rec;
  dim3 grid(A.n_splits * A.n_rt, dm.Hkv, dm.B), cgrid(A.n_rt, dm.Hkv, dm.B);
  if (dm.D == 64) {
    if (kv_fp8) hipLaunchKernelGGL((k_attn_decode<64, true>), grid, dim3(256), 0, s, A);
    else hipLaunchKernelGGL((k_attn_decode<64, false>), grid, dim3(256), 0, s, A);
    if (A.n_splits > 1) hipLaunchKernelGGL(k_attn_combine<64>, cgrid, dim3(256), 0, s, A);
  } else {
    if (kv_fp8) hipLaunchKernelGGL((k_attn_decode<128, true>), grid, dim3(256), 0, s, A);
    else hipLaunchKernelGGL((k_attn_decode<128, false>), grid, dim3(256), 0, s, A);
    if (A.n_splits > 1) hipLaunchKernelGGL(k_attn_combine<128>, cgrid, dim3(256), 0, s, A);
  }
}

}  // namespace plt
