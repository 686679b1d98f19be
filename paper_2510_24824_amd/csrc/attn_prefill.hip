// Prefill attention on gfx950 matrix cores (bf16 storage, float statistics): the token-parallel
// form of the PLT attention [Alg. 2 forward; Alg. 3 l.2-5 for loops >= 2].
//
//   loop 1      : y[p] = Attn(q[p], K_share[0..p], V_share[0..p])                 (causal)
//   loops >= 2  : y[p] = g * Attn(q[p], K_own[p-w+1..p], V_own[..]) + (1-g) * Attn(q[p], K_share[0..p], ..)
//
// A workgroup owns 128 consecutive positions of one query head: 4 waves x 2 tiles of 16 query
// rows.  Key/value tiles of 32 positions are copied once per workgroup from the cache into LDS
// (next tile prefetched into registers meanwhile) and every fragment a wave reads from LDS feeds
// both of its query tiles, so a K/V byte fetched from L2 is used by 128 query rows.  The tile
// algebra is the decode kernel's: S^T = K Q^T, O^T += V^T P^T with v_mfma_f32_16x16x32_bf16, one
// query row per lane in S^T, P^T and O^T, row maxima via two wavefront shuffles.  A wave owns its
// rows for the whole key range, so no cross-wave merge is needed.
// e4m3 caches (F8): the bytes are expanded to bf16 (exactly) on their way into LDS; the rest is shared.
#include "plt_internal.h"

namespace plt {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) float f32x8;

namespace {

constexpr int PF_QROWS = 128;                 // query positions per workgroup
#define PF_NEG_INF (-INFINITY)
#define PF_M_INIT (-1.0e30f)

__device__ inline bf16x8 pf_bf(uint4 v) { return __builtin_bit_cast(bf16x8, v); }

template <int D>
struct PfState {           // online softmax state of one 16-row query tile
  float m;                 // running maximum (log2 domain); starts at a large negative finite value, so that
                           // m - m is 0 and not NaN for rows that have attended nothing yet
  f32x4 l;                 // softmax denominator: every element holds the row's full sum (see pf_tile)
  f32x4 acc[D / 16];
  __device__ void init() {
    m = PF_M_INIT; l = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < D / 16; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
};

// LDS tile of 32 keys.  16-byte chunks are XOR-swizzled so that the eight lanes the LDS serves together
// (same chunk column, rows 0-3 and 8-11 of a K sub-tile, or eight consecutive V rows of 64 bytes) fall
// into eight different bank groups.
template <int D>
struct PfLds {
  bf16_t k[32][D];         // [key][feature]; chunk c of row r at chunk c ^ kx(r)
  bf16_t v[D][32];         // [feature][position]; chunk c of row d at chunk c ^ ((d >> 1) & 3)
  // kx: distinct over the eight rows a fragment read serves together (r, r+1, r+2, r+3, r+8 .. r+11) AND with bit 2
  // differing between the two consecutive rows whose chunks 0..3 one group of eight lanes writes when a tile is
  // stored (with r % 4 in the low bits those two rows' chunks fell into the same four bank groups: two-way conflicts)
  __device__ static int kx(int r) { return ((r & 1) << 2) | ((r >> 1) & 1) | (((r >> 3) & 1) << 1); }
  __device__ bf16_t* kp(int r, int c) { return &k[r][(c ^ kx(r)) * 8]; }
  __device__ const bf16_t* kp(int r, int c) const { return &k[r][(c ^ kx(r)) * 8]; }
  __device__ bf16_t* vp(int d, int c) { return &v[d][(c ^ ((d >> 1) & 3)) * 8]; }
  __device__ const bf16_t* vp(int d, int c) const { return &v[d][(c ^ ((d >> 1) & 3)) * 8]; }
};

// Online-softmax update of one 16-row query tile for a 64-key tile made of two 32-key halves: s[h][a] are the
// raw scores of half h, 16-key sub-tile a (this lane: keys 32h + 8g + 4a + i of the tile).  Returns the bf16
// probabilities per half (B operands of the second contraction) and rescales the accumulators when some row's
// maximum moved.  Key j is attended iff lo < j <= hi.
template <int D>
__device__ __forceinline__ void pf_softmax(PfState<D>& st, const f32x4 (&s)[2][2], float scale_log2, int key_base,
                                           bool need_mask, int lo, int hi, int g, bf16x8 (&pb)[2]) {
  float sv[16];
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int i = 0; i < 4; ++i) { sv[8 * h + i] = s[h][0][i]; sv[8 * h + 4 + i] = s[h][1][i]; }
  if (need_mask) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int kb = key_base + 32 * h + 8 * g;
#pragma unroll
      for (int j = 0; j < 8; ++j) if (kb + j > hi || kb + j <= lo) sv[8 * h + j] = PF_NEG_INF;
    }
  }
  float mx = sv[0];
#pragma unroll
  for (int j = 1; j < 16; ++j) mx = fmaxf(mx, sv[j]);
  mx = row4_max_f32(mx);
  const float m_new = fmaxf(st.m, mx * scale_log2);        // the scale is positive: max and scaling commute
  const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
  f32x8 p[2];
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int j = 0; j < 8; ++j) p[h][j] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[8 * h + j], scale_log2, -m_new));
  st.m = m_new;
  // alpha == 1 in every lane (no row of this tile raised its maximum: the usual case after the first
  // few tiles): the rescale of the accumulators is skipped for the whole wave
  if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
      st.acc[dt][0] *= alpha; st.acc[dt][1] *= alpha; st.acc[dt][2] *= alpha; st.acc[dt][3] *= alpha;
    }
    st.l[0] *= alpha; st.l[1] *= alpha; st.l[2] *= alpha; st.l[3] *= alpha;
  }
  pb[0] = __builtin_convertvector(p[0], bf16x8); pb[1] = __builtin_convertvector(p[1], bf16x8);
}

// One 64-key tile (two 32-key halves in LDS) for the two query tiles of a wave.  lo/hi: per lane (= per query
// row) bounds.  One softmax step per 64 keys: its fixed cost (row maximum across lanes, rescale test, state
// update) is paid half as often as with 32-key steps, and the vector ALU is what bounds this kernel.
template <int D>
__device__ __forceinline__ void pf_tile(PfState<D> (&st)[2], const PfLds<D> (&sm)[2], const uint4 (&qf)[2][D / 32],
                               float scale_log2, int key_base, bool need_mask, const int (&lo)[2],
                               const int (&hi)[2], int m16, int g) {
  const int key0 = 8 * (m16 >> 2) + (m16 & 3);
  f32x4 s[2][2][2];                 // [query tile][half][sub-tile]
#pragma unroll
  for (int q = 0; q < 2; ++q)
#pragma unroll
    for (int h = 0; h < 2; ++h) { s[q][h][0] = f32x4{0.f, 0.f, 0.f, 0.f}; s[q][h][1] = f32x4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
      const uint4 k0 = *reinterpret_cast<const uint4*>(sm[h].kp(key0, kk * 4 + g));
      const uint4 k1 = *reinterpret_cast<const uint4*>(sm[h].kp(key0 + 4, kk * 4 + g));
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        s[q][h][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf_bf(k0), pf_bf(qf[q][kk]), s[q][h][0], 0, 0, 0);
        s[q][h][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf_bf(k1), pf_bf(qf[q][kk]), s[q][h][1], 0, 0, 0);
      }
    }
  bf16x8 pb[2][2];
#pragma unroll
  for (int q = 0; q < 2; ++q) pf_softmax<D>(st[q], s[q], scale_log2, key_base, need_mask, lo[q], hi[q], g, pb[q]);
  // the softmax denominators come from the matrix cores as well: a block of ones in place of V^T sums the (bf16)
  // probabilities over the 32 keys of a half, into every element of l
  const uint4 ones = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int q = 0; q < 2; ++q) st[q].l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf_bf(ones), pb[q][h], st[q].l, 0, 0, 0);
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
      const uint4 vf = *reinterpret_cast<const uint4*>(sm[h].vp(dt * 16 + m16, g));
#pragma unroll
      for (int q = 0; q < 2; ++q)
        st[q].acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf_bf(vf), pb[q][h], st[q].acc[dt], 0, 0, 0);
    }
}

struct PfArgs {
  const bf16_t* q; const float* z; bf16_t* y;
  float* tmp;      // [rows, Hq*D] float: g * y_local parked between the two passes (gated rows only)
  const char* k_share; const char* v_share; const char* k_loc; const char* v_loc;   // bf16 or e4m3 elements
  int n, n_pad, n_pad_loc, w, b0, Hq, Hkv, G, gated, n_qt, Bc;
  float scale_log2;
};

// Streams the 32-key blocks t_beg..t_end-1 of one K/V stream (n_blk blocks are allocated) through LDS, two
// blocks (64 keys) per step, and applies them to the wave's two query tiles; a block outside the range that
// shares a step with one inside is masked by the rows' bounds.
// All 256 threads of the workgroup must call this together.
template <int D, bool F8>
__device__ __forceinline__ void pf_pass(PfState<D> (&st)[2], PfLds<D> (&sm)[2], const char* __restrict__ kbase,
                               const char* __restrict__ vbase, int t_beg, int t_end, int n_blk, const uint4 (&qf)[2][D / 32],
                               float scale_log2, const int (&lo)[2], const int (&hi)[2], int row_min, int row_max,
                               int m16, int g) {
  const int tid = threadIdx.x;
  constexpr int ES = F8 ? 1 : 2;
  constexpr int TILE_BYTES = 32 * D * ES;                       // of a block's K tile and of its V block alike
  constexpr int KCH = (TILE_BYTES / 16 + 255) / 256;            // 16-byte chunks per thread and block (1 or 2)
  constexpr int NCH = TILE_BYTES / 16;                          // chunks per block (may be < 256)
  // register staging of the next step (plain loops: the arrays must stay in registers)
  uint4 rk[2][KCH], rv[2][KCH];
#pragma unroll
  for (int i = 0; i < KCH; ++i) { rk[0][i] = rk[1][i] = make_uint4(0, 0, 0, 0); rv[0][i] = rv[1][i] = make_uint4(0, 0, 0, 0); }
  // The cache keeps K in the decode kernel's load order (kblk_index): a 16-byte chunk of a block is
  // (sub-tile a, feature chunk kk, row m, lane group g) and belongs to key kkey, features kcol ..; its address
  // is a block offset (the same for all threads: scalar registers) plus a per-thread constant koff.
  auto k_chunk = [&](int h, int ch, unsigned& koff, int& kkey, int& kcol) {
    if (F8) {   // 64-key blocks; the 32-key block is half h of one: rows m with (m >> 2) in {2h, 2h+1}
      const int g = ch & 3, m = 8 * h + ((ch >> 2) & 7), kk = (ch >> 5) % (D / 64), a = (ch >> 5) / (D / 64);
      koff = (unsigned)(((a * (D / 64) + kk) * 64 + m * 4 + g) * 16);
      kkey = 16 * ((m >> 2) & 1) + (m & 3) + 4 * a; kcol = kk * 64 + g * 16;
    } else {
      const int g = ch & 3, m = (ch >> 2) & 15, kk = (ch >> 6) % (D / 32), a = (ch >> 6) / (D / 32);
      koff = (unsigned)ch * 16u;
      kkey = 8 * (m >> 2) + (m & 3) + 4 * a; kcol = kk * 32 + g * 8;
    }
  };
  auto fetch = [&](int T) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      // a block beyond the allocation is replaced by the last allocated one (finite values; its keys lie
      // beyond every row's bound and are masked)
      const int t = (2 * T + h < n_blk) ? 2 * T + h : n_blk - 1;          // the same for all threads
      const char* kt = kbase + (F8 ? (size_t)(t >> 1) * 64 * D : (size_t)t * TILE_BYTES);
      const char* vt = vbase + (size_t)t * TILE_BYTES;
#pragma unroll
      for (int i = 0; i < KCH; ++i) {
        const int ch = tid + i * 256;
        if (NCH % 256 == 0 || ch < NCH) {
          unsigned koff; int kkey, kcol;
          k_chunk(F8 ? (t & 1) : h, ch, koff, kkey, kcol);
          rk[h][i] = *reinterpret_cast<const uint4*>(kt + koff);
          rv[h][i] = *reinterpret_cast<const uint4*>(vt + (unsigned)ch * 16u);
        }
      }
    }
  };
  // staged registers -> LDS (e4m3 bytes are expanded to bf16 here)
  auto store = [&]() {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      PfLds<D>& dst = sm[h];
#pragma unroll
      for (int i = 0; i < KCH; ++i) {
        const int ch = tid + i * 256;
        if (NCH % 256 == 0 || ch < NCH) {
          unsigned koff; int kkey, kcol;
          k_chunk(h, ch, koff, kkey, kcol);
          if (F8) {
            *reinterpret_cast<bf16x8*>(dst.kp(kkey, kcol / 8)) = e4m3x8_to_bf16(rk[h][i].x, rk[h][i].y);
            *reinterpret_cast<bf16x8*>(dst.kp(kkey, kcol / 8 + 1)) = e4m3x8_to_bf16(rk[h][i].z, rk[h][i].w);
            // V chunk ch of the block = (feature group ch / 32, position half (ch / 16) % 2, feature ch % 16)
            const int vd = (ch >> 5) * 16 + (ch & 15), vc = ((ch >> 4) & 1) * 2;
            *reinterpret_cast<bf16x8*>(dst.vp(vd, vc)) = e4m3x8_to_bf16(rv[h][i].x, rv[h][i].y);
            *reinterpret_cast<bf16x8*>(dst.vp(vd, vc + 1)) = e4m3x8_to_bf16(rv[h][i].z, rv[h][i].w);
          } else {
            *reinterpret_cast<uint4*>(dst.kp(kkey, kcol / 8)) = rk[h][i];
            // V chunk ch of the block = (feature group ch / 64, position chunk (ch / 16) % 4, feature ch % 16)
            *reinterpret_cast<uint4*>(dst.vp((ch >> 6) * 16 + (ch & 15), (ch >> 4) & 3)) = rv[h][i];
          }
        }
      }
    }
  };
  const int T_beg = t_beg >> 1, T_end = (t_end + 1) >> 1;
  const int lo_max = __builtin_amdgcn_readlane(lo[1], 15);      // the wave's last row has the largest lower bound
  if (T_beg < T_end) fetch(T_beg);
  for (int T = T_beg; T < T_end; ++T) {
    __syncthreads();                         // every wave is done with the previous step
    store();
    __syncthreads();
    if (T + 1 < T_end) fetch(T + 1);
    const int kb = T * 64;
    // Every wave multiplies every step of the workgroup's range, also the few that none of its rows may
    // attend (they are masked out entirely): skipping them made the accumulators take two paths through
    // the loop, which cost a copy of all 64 accumulator registers per step.  Steps that straddle a bound
    // of some row are masked, the others are not.
    const bool need_mask = (kb + 63 > row_min) || (kb <= lo_max);
    pf_tile<D>(st, sm, qf, scale_log2, kb, need_mask, lo, hi, m16, g);
  }
}

template <int D, bool F8>
__global__ __launch_bounds__(256, 2) void k_attn_prefill2(PfArgs A) {
  constexpr int ES = F8 ? 1 : 2;
  __shared__ __attribute__((aligned(16))) PfLds<D> sm[2];      // the two 32-key halves of a step
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, m16 = lane & 15, g = lane >> 4;
  // Workgroups are dispatched in blockIdx.x order: all (head, sequence) pairs of the query tile with
  // the longest key range first, the shortest ranges last, so the causal imbalance does not leave a
  // few long workgroups running alone at the end.
  const int hb = (int)blockIdx.x % (A.Hq * A.Bc);
  const int qt = A.n_qt - 1 - (int)blockIdx.x / (A.Hq * A.Bc);
  const int h = hb % A.Hq, b = hb / A.Hq, kvh = h / A.G;
  const int p0 = qt * PF_QROWS;
  const int p_last = (p0 + PF_QROWS - 1 < A.n ? p0 + PF_QROWS - 1 : A.n - 1);
  // this lane's two query rows
  int prow[2], hi[2], lo_g[2], lo_l[2];
  uint4 qf[2][D / 32];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    prow[q] = p0 + wv * 32 + q * 16 + m16;
    const bool ok = prow[q] < A.n;
    hi[q] = ok ? prow[q] : -1;                         // rows beyond the prompt attend nothing
    lo_g[q] = -1;
    lo_l[q] = prow[q] - A.w;                           // monotone in the row, also for rows beyond the prompt
#pragma unroll
    for (int kk = 0; kk < D / 32; ++kk) {
      qf[q][kk] = make_uint4(0, 0, 0, 0);
      if (ok) qf[q][kk] = *reinterpret_cast<const uint4*>(A.q + (((size_t)b * A.n + prow[q]) * A.Hq + h) * D + kk * 32 + g * 8);
    }
  }
  const int row_min = p0 + wv * 32, row_max_raw = p0 + wv * 32 + 31;
  const int row_max = row_max_raw < A.n ? row_max_raw : A.n - 1;

  // One softmax state is live at a time: the window pass runs first and parks g * y_local (float)
  // in a scratch row that the same lane reads back in the epilogue of the global pass.
  PfState<D> st[2];
  float gate[2] = {0.f, 0.f};
  if (A.gated) {
    st[0].init(); st[1].init();
    const size_t stream = (size_t)b * A.Hkv + kvh;
    int j_lo = p0 - A.w + 1; if (j_lo < 0) j_lo = 0;
    pf_pass<D, F8>(st, sm, A.k_loc + stream * (size_t)A.n_pad_loc * D * ES, A.v_loc + stream * (size_t)A.n_pad_loc * D * ES,
               j_lo >> 5, (p_last >> 5) + 1, A.n_pad_loc >> 5, qf, A.scale_log2, lo_l, hi, row_min, row_max, m16, g);
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      if (prow[q] >= A.n) continue;
      const float ll = st[q].l[0];
      const size_t r = (size_t)b * A.n + prow[q];
      gate[q] = 1.0f / (1.0f + __expf(-A.z[r * A.Hq + h]));
      const float f = ll > 0.f ? gate[q] / ll : 0.f;
      float* dst = A.tmp + (r * A.Hq + h) * D;
#pragma unroll
      for (int dt = 0; dt < D / 16; ++dt) {
        f32x4 v = st[q].acc[dt];
        v[0] *= f; v[1] *= f; v[2] *= f; v[3] *= f;
        *reinterpret_cast<f32x4*>(dst + dt * 16 + 4 * g) = v;
      }
    }
  }
  st[0].init(); st[1].init();
  {
    const size_t stream = (size_t)(A.b0 + b) * A.Hkv + kvh;
    pf_pass<D, F8>(st, sm, A.k_share + stream * (size_t)A.n_pad * D * ES, A.v_share + stream * (size_t)A.n_pad * D * ES, 0,
               (p_last >> 5) + 1, A.n_pad >> 5, qf, A.scale_log2, lo_g, hi, row_min, row_max, m16, g);
  }
  // epilogue: lane (row m16, g) holds features dt*16 + 4g .. +3 of its two rows
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    if (prow[q] >= A.n) continue;
    const float lg = st[q].l[0];
    const float fg = (lg > 0.f ? 1.0f / lg : 0.f) * (1.0f - gate[q]);     // gate = 0 for first-loop rows
    const size_t r = (size_t)b * A.n + prow[q];
    bf16_t* dst = A.y + (r * A.Hq + h) * D;
    const float* loc = A.tmp + (r * A.Hq + h) * D;
#pragma unroll
    for (int dt = 0; dt < D / 16; ++dt) {
      f32x4 v = st[q].acc[dt];
      v[0] *= fg; v[1] *= fg; v[2] *= fg; v[3] *= fg;
      if (A.gated) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(loc + dt * 16 + 4 * g);
        v[0] += t[0]; v[1] += t[1]; v[2] += t[2]; v[3] += t[3];
      }
      ushort4 o;
      o.x = f32_to_bf16(v[0]); o.y = f32_to_bf16(v[1]); o.z = f32_to_bf16(v[2]); o.w = f32_to_bf16(v[3]);
      *reinterpret_cast<ushort4*>(dst + dt * 16 + 4 * g) = o;
    }
  }
}

}  // namespace

void launch_attn_prefill_mfma(hipStream_t s, const bf16_t* q, const float* z, bf16_t* y, float* local_tmp,
                              KvView kv, int Bc, int n, int loop, Dims dm, int plain, int kv_fp8) {
  PfArgs A;
  A.q = q; A.z = z; A.y = y; A.tmp = local_tmp;
  A.k_share = (const char*)kv.k_share; A.v_share = (const char*)kv.v_share;
  A.k_loc = (const char*)kv.k_loc; A.v_loc = (const char*)kv.v_loc;
  A.n = n; A.n_pad = kv.n_pad; A.n_pad_loc = kv.n_pad_loc; A.w = kv.w; A.b0 = kv.b0;
  A.Hq = dm.Hq; A.Hkv = dm.Hkv; A.G = dm.Hq / dm.Hkv;
  A.gated = (!plain && loop > 0) ? 1 : 0;
  A.n_qt = (n + PF_QROWS - 1) / PF_QROWS;
  A.scale_log2 = 1.4426950408889634f / sqrtf((float)dm.D);
  A.Bc = Bc;
  dim3 grid((unsigned)A.n_qt * dm.Hq * Bc);
  if (dm.D == 64) {
    if (kv_fp8) hipLaunchKernelGGL((k_attn_prefill2<64, true>), grid, dim3(256), 0, s, A);
    else hipLaunchKernelGGL((k_attn_prefill2<64, false>), grid, dim3(256), 0, s, A);
  } else {
    if (kv_fp8) hipLaunchKernelGGL((k_attn_prefill2<128, true>), grid, dim3(256), 0, s, A);
    else hipLaunchKernelGGL((k_attn_prefill2<128, false>), grid, dim3(256), 0, s, A);
  }
}

}  // namespace plt
