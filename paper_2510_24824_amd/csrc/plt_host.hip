// Host side of libplt.so: the C ABI of include/plt.h, the cache / weight layouts and the
// CLP token/loop scheduler (which kernels run, in which order, on which rows).
#include <hip/hip_runtime.h>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>
#include "plt_internal.h"

using namespace plt;

// ------------------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";
static int fail(int code, const char* fmt, ...) {
  va_list ap; va_start(ap, fmt); vsnprintf(g_err, sizeof(g_err), fmt, ap); va_end(ap);
  return code;
}
#define HIP_TRY(expr)                                                                     \
  do { hipError_t e_ = (expr);                                                            \
       if (e_ != hipSuccess) return fail(PLT_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); } while (0)

extern "C" const char* plt_last_error(void) { return g_err; }

// ------------------------------------------------------------------------------ static scratch
// Device memory the library itself holds, for the entry point that must not allocate
// (plt_attn_decode_static): the split partials of the fused decode attention live here.  Every GPU the library
// runs on holds its own copy of the array until the process ends.  In host code the array's NAME is only a
// stand-in: the device address comes from hipGetSymbolAddress, once per device with that device current, and
// only that pointer is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[PLT_ATTN_STATIC_SCRATCH_BYTES];
static const int MAX_DEVICES = 64;
static void* g_scratch_ptr[MAX_DEVICES];     // per device: address of that device's copy of `scratch`, or null
static std::mutex g_scratch_mu;
static int static_scratch(void** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(PLT_EINVAL, "static scratch: device index %d not supported", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(PLT_EHIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return PLT_OK;
}

// ------------------------------------------------------------------------------ objects
struct LayerW {
  const float* norm1; const void* wqkv; const float* gate_w; const float* gate_b;
  const void* wo; const float* norm2; const void* wgu; const void* wdown;
  const void* router;   // mixture-of-experts models only
  const uint8_t *wqkv_sc, *wo_sc, *wgu_sc, *wdown_sc;   // low-bit models: block scales of the four projections
};
struct ProfRec { hipEvent_t a, b; int klass; };
struct plt_model {
  int profile = 0;   // bit mask of instrumented launch classes (1 << PLT_PROF_*)
  std::vector<ProfRec> prof_used, prof_free;
  plt_config cfg;
  hipStream_t stream;
  const char* blob;
  std::vector<LayerW> layers;
  const void* emb; const float* norm_f; const void* head;
  int es;   // element size of the model dtype
  int kes;  // element size of the caches (es, or 1 for e4m3 caches)
  bool kv8; // caches hold e4m3 bytes
  bool mx;  // the four per-layer projections run on MXFP4 weights and MXFP8 activations
  double* inv_freq = nullptr;   // device [D/2]: rotary frequencies theta^(-2j/D), computed in double
  bool use_graph = false;       // plt_decode_step replays its launch sequence as a HIP graph (see plt_use_graph)
  int phys_layers = 0;          // timing-only aliasing of the shared caches: layer m uses the memory of layer m % phys_layers (0: off)
};
struct plt_kv {
  plt_model* m;
  int B, max_ctx, n_pad, w_pad, n_caches, n_rings;
  int share_layers;    // layers of shared cache physically present (= n_layers unless aliased for timing)
  char* buf;
  size_t share_elems;  // elements of one layer's K_share (= V_share): B*Hkv*n_pad*D
  size_t ring_elems;   // elements of one layer's ring K (= ring V): B*(L-1)*Hkv*w_pad*D
  size_t ring_base;    // byte offset of the ring area
  int pos; bool started;
  // per-step activation scratch (device, library-owned)
  float* x; void* a; float* gout; size_t gout_elems; void* q; float* z; void* y; void* act;
  float* carry; int32_t* pos_dev; void* attn_scratch; size_t attn_scratch_bytes;
  void* moe_idx;       // mixture-of-experts models: routing lists of one pass (moe_index_bytes)
  uint8_t *a_codes, *a_scales;   // low-bit models: the quantised input of the next projection
  uint8_t* act_sc;               // low-bit mixture-of-experts models: block scales of the experts' hidden rows
  float* arg_v; int* arg_i;   // argmax chunk winners
  // test hook (plt_debug_layer on a low-bit model): copies of the e4m3 codes / block scales that entered the layer's
  // four projections, one slot per projection (allocated on first use)
  uint8_t* dbg_codes = nullptr; uint8_t* dbg_scales = nullptr; size_t dbg_codes_slot = 0, dbg_scales_slot = 0; bool dbg_on = false;
  // the decode step's launch sequence as an instantiated HIP graph, valid for these arguments / this split count
  hipGraphExec_t graph_exec = nullptr;
  const int32_t* g_tokens = nullptr; int32_t* g_next = nullptr; float* g_logits = nullptr; int g_splits = -1;
};

static bool cfg_valid(const plt_config* c, const char** why) {
  *why = "";
  if (!c) { *why = "null config"; return false; }
  if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->n_kv_heads < 1 || c->ffn_hidden < 1 ||
      c->vocab < 1) { *why = "non-positive dimension"; return false; }
  if (c->head_dim != 64 && c->head_dim != 128) { *why = "head_dim must be 64 or 128"; return false; }
  if (c->n_heads % c->n_kv_heads) { *why = "n_heads must be a multiple of n_kv_heads"; return false; }
  if (c->n_loops < 1 || c->n_loops > 16) { *why = "n_loops must be in 1..16"; return false; }
  if (c->mode != PLT_MODE_CLP && c->mode != PLT_MODE_VANILLA_LOOP && c->mode != PLT_MODE_CLP_SHARE_ONLY &&
      c->mode != PLT_MODE_CLP_OWN_KV) { *why = "unknown mode"; return false; }
  if (c->mode == PLT_MODE_CLP && c->n_loops > 1 && c->window < 1) { *why = "window must be >= 1"; return false; }
  if (c->dtype != PLT_F32 && c->dtype != PLT_BF16) { *why = "unknown dtype"; return false; }
  if (c->dtype == PLT_BF16 && (c->d_model % 64 || c->ffn_hidden % 64)) {
    *why = "bf16 needs d_model and ffn_hidden to be multiples of 64"; return false;
  }
  if (!(c->rope_theta > 0.f) || !(c->norm_eps >= 0.f)) { *why = "bad rope_theta / norm_eps"; return false; }
  if (c->kv_dtype != 0 && c->kv_dtype != PLT_FP8_E4M3) { *why = "unknown kv_dtype"; return false; }
  if (c->kv_dtype == PLT_FP8_E4M3 && c->dtype != PLT_BF16) { *why = "e4m3 caches need dtype PLT_BF16"; return false; }
  if (c->w_dtype != 0 && c->w_dtype != PLT_MXFP4) { *why = "unknown w_dtype"; return false; }
  if (c->w_dtype == PLT_MXFP4) {
    if (c->dtype != PLT_BF16) { *why = "MXFP4 projections need dtype PLT_BF16"; return false; }
    if (c->d_model % 128 || c->ffn_hidden % 128 || (c->n_heads * c->head_dim) % 128) {
      *why = "MXFP4 projections need d_model, ffn_hidden and n_heads * head_dim to be multiples of 128"; return false;
    }
  }
  if (c->n_experts < 0 || c->n_experts > 256) { *why = "n_experts must be in 0..256"; return false; }
  if (c->n_experts > 0 && (c->top_k < 1 || c->top_k > c->n_experts || c->top_k > 32)) {
    *why = "top_k must be in 1..min(n_experts, 32)"; return false;
  }
  return true;
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// walks the blob layout; returns total bytes, reports one tensor if asked
static size_t blob_walk(const plt_config* c, int want_layer, int want_which, size_t* off, size_t* nelem) {
  const size_t es = c->dtype == PLT_BF16 ? 2 : 4;
  const size_t d = c->d_model, Hq = c->n_heads, Hkv = c->n_kv_heads, D = c->head_dim, F = c->ffn_hidden,
               V = c->vocab, E = c->n_experts, Ex = E > 0 ? E : 1;
  size_t cur = 0;
  auto put = [&](int layer, int which, size_t n, size_t esz) {
    cur = align256(cur);
    if (which == want_which && (layer == want_layer || layer < 0)) { if (off) *off = cur; if (nelem) *nelem = n; }
    cur += n * esz;
  };
  // low-bit projection [N, K]: e2m1 codes (reported element count N*K, two per byte), then its scale bytes
  const bool mx = c->w_dtype == PLT_MXFP4;
  auto put_w = [&](int layer, int which, int which_sc, size_t N, size_t K, size_t count = 1) {   // count matrices back to back
    if (!mx) { put(layer, which, count * N * K, es); return; }
    cur = align256(cur);
    if (which == want_which && layer == want_layer) { if (off) *off = cur; if (nelem) *nelem = count * N * K; }
    cur += count * N * K / 2;
    cur = align256(cur);
    const size_t sb = count * mx_wscale_bytes((int)N, (int)K);
    if (which_sc == want_which && layer == want_layer) { if (off) *off = cur; if (nelem) *nelem = sb; }
    cur += sb;
  };
  put(-1, PLT_W_EMB, V * d, es);
  for (int m = 0; m < c->n_layers; ++m) {
    put(m, PLT_W_NORM1, d, 4);
    put_w(m, PLT_W_WQKV, PLT_W_WQKV_SC, (Hq + 2 * Hkv) * D, d);
    put(m, PLT_W_GATE_W, Hq * D, 4);
    put(m, PLT_W_GATE_B, Hq, 4);
    put_w(m, PLT_W_WO, PLT_W_WO_SC, d, Hq * D);
    put(m, PLT_W_NORM2, d, 4);
    if (E > 0) put(m, PLT_W_ROUTER, E * d, es);
    if (mx) { put_w(m, PLT_W_WGU, PLT_W_WGU_SC, 2 * F, d, Ex); put_w(m, PLT_W_WDOWN, PLT_W_WDOWN_SC, d, F, Ex); }
    else { put(m, PLT_W_WGU, Ex * 2 * F * d, es); put(m, PLT_W_WDOWN, Ex * d * F, es); }
  }
  put(-1, PLT_W_NORM_F, d, 4);
  if (!c->tie_embeddings) put(-1, PLT_W_HEAD, V * d, es);
  return align256(cur);
}

extern "C" size_t plt_weights_bytes(const plt_config* cfg) {
  const char* why;
  if (!cfg_valid(cfg, &why)) { fail(PLT_EINVAL, "plt_weights_bytes: %s", why); return 0; }
  return blob_walk(cfg, -2, -1, nullptr, nullptr);
}

extern "C" int plt_weights_offset(const plt_config* cfg, int32_t layer, int32_t which, size_t* off,
                                  size_t* nelem) {
  const char* why;
  if (!cfg_valid(cfg, &why)) return fail(PLT_EINVAL, "plt_weights_offset: %s", why);
  if (which < PLT_W_EMB || which > PLT_W_WDOWN_SC || !off || !nelem) return fail(PLT_EINVAL, "plt_weights_offset: bad tensor id or null output");
  const bool global = which == PLT_W_EMB || which == PLT_W_NORM_F || which == PLT_W_HEAD;
  if (which == PLT_W_HEAD && cfg->tie_embeddings) return fail(PLT_EINVAL, "plt_weights_offset: head is tied to the embedding");
  if (which == PLT_W_ROUTER && cfg->n_experts == 0) return fail(PLT_EINVAL, "plt_weights_offset: a dense model has no router");
  if (which >= PLT_W_WQKV_SC && cfg->w_dtype != PLT_MXFP4) return fail(PLT_EINVAL, "plt_weights_offset: only MXFP4 models have scale tensors");
  if (!global && (layer < 0 || layer >= cfg->n_layers)) return fail(PLT_EINVAL, "plt_weights_offset: layer out of range");
  *off = (size_t)-1;
  blob_walk(cfg, global ? -1 : layer, which, off, nelem);
  if (*off == (size_t)-1) return fail(PLT_EINVAL, "plt_weights_offset: tensor not found");
  return PLT_OK;
}

extern "C" int plt_init(const plt_config* cfg, const void* dev_weights, size_t nbytes, void* hip_stream,
                        plt_model** out) {
  const char* why;
  if (!out) return fail(PLT_EINVAL, "plt_init: null output pointer");
  *out = nullptr;
  if (!cfg_valid(cfg, &why)) return fail(PLT_EINVAL, "plt_init: %s", why);
  if (!dev_weights) return fail(PLT_EINVAL, "plt_init: null weight blob");
  const size_t need = blob_walk(cfg, -2, -1, nullptr, nullptr);
  if (nbytes < need) return fail(PLT_ENOMEM, "plt_init: weight blob has %zu bytes, layout needs %zu", nbytes, need);
  if (((uintptr_t)dev_weights) & 255) return fail(PLT_EINVAL, "plt_init: weight blob must be 256-byte aligned");
  int ndev = 0;
  HIP_TRY(hipGetDeviceCount(&ndev));
  {
    // set-up time is when the current device's copy of the static scratch is looked up (plt_attn_decode_static
    // does it on its first call on a device otherwise)
    void* sp = nullptr;
    const int rc = static_scratch(&sp);
    if (rc != PLT_OK) return rc;
  }
  plt_model* m = new (std::nothrow) plt_model();
  if (!m) return fail(PLT_ENOMEM, "plt_init: out of host memory");
  m->cfg = *cfg; m->stream = (hipStream_t)hip_stream; m->blob = (const char*)dev_weights;
  m->es = cfg->dtype == PLT_BF16 ? 2 : 4;
  m->kv8 = cfg->kv_dtype == PLT_FP8_E4M3;
  m->kes = m->kv8 ? 1 : m->es;
  m->mx = cfg->w_dtype == PLT_MXFP4;
  auto at = [&](int layer, int which) -> const void* {
    size_t off = 0, n = 0; blob_walk(cfg, layer, which, &off, &n); return m->blob + off;
  };
  m->emb = at(-1, PLT_W_EMB);
  m->norm_f = (const float*)at(-1, PLT_W_NORM_F);
  m->head = cfg->tie_embeddings ? m->emb : at(-1, PLT_W_HEAD);
  m->layers.resize(cfg->n_layers);
  for (int l = 0; l < cfg->n_layers; ++l) {
    LayerW& w = m->layers[l];
    w.norm1 = (const float*)at(l, PLT_W_NORM1); w.wqkv = at(l, PLT_W_WQKV);
    w.gate_w = (const float*)at(l, PLT_W_GATE_W); w.gate_b = (const float*)at(l, PLT_W_GATE_B);
    w.wo = at(l, PLT_W_WO); w.norm2 = (const float*)at(l, PLT_W_NORM2);
    w.wgu = at(l, PLT_W_WGU); w.wdown = at(l, PLT_W_WDOWN);
    w.router = cfg->n_experts > 0 ? at(l, PLT_W_ROUTER) : nullptr;
    w.wqkv_sc = w.wo_sc = w.wgu_sc = w.wdown_sc = nullptr;
    if (m->mx) {
      w.wqkv_sc = (const uint8_t*)at(l, PLT_W_WQKV_SC); w.wo_sc = (const uint8_t*)at(l, PLT_W_WO_SC);
      w.wgu_sc = (const uint8_t*)at(l, PLT_W_WGU_SC); w.wdown_sc = (const uint8_t*)at(l, PLT_W_WDOWN_SC);
    }
  }
  {
    std::vector<double> f(cfg->head_dim / 2);
    for (int j = 0; j < cfg->head_dim / 2; ++j) f[j] = std::pow((double)cfg->rope_theta, -2.0 * j / cfg->head_dim);
    hipError_t e = hipMalloc((void**)&m->inv_freq, f.size() * sizeof(double));
    if (e == hipSuccess) e = hipMemcpy(m->inv_freq, f.data(), f.size() * sizeof(double), hipMemcpyHostToDevice);
    if (e != hipSuccess) { if (m->inv_freq) (void)hipFree(m->inv_freq); delete m; return fail(PLT_EHIP, "plt_init: %s", hipGetErrorString(e)); }
  }
  *out = m;
  return PLT_OK;
}

extern "C" void plt_free(plt_model* m) {
  if (!m) return;
  if (m->inv_freq) (void)hipFree(m->inv_freq);
  for (auto* v : {&m->prof_used, &m->prof_free})
    for (ProfRec& r : *v) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  delete m;
}

// ---- bench instrumentation: event pairs around selected launches ----
struct ProfScope {
  plt_model* m; ProfRec r; bool on;
  ProfScope(plt_model* m_, int klass, bool decode) : m(m_), on(((m_->profile >> klass) & 1) && decode) {
    if (!on) return;
    if (!m->prof_free.empty()) { r = m->prof_free.back(); m->prof_free.pop_back(); }
    else if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) { on = false; return; }
    r.klass = klass;
    (void)hipEventRecord(r.a, m->stream);
  }
  ~ProfScope() { if (on) { (void)hipEventRecord(r.b, m->stream); m->prof_used.push_back(r); } }
};

extern "C" int plt_profile_enable(plt_model* m, int32_t on) {
  if (!m) return fail(PLT_EINVAL, "plt_profile_enable: null model");
  m->profile = on;
  return PLT_OK;
}

extern "C" int plt_profile_read(plt_model* m, int32_t klass, double* ms_sum, int64_t* launches, int32_t reset) {
  if (!m || !ms_sum || !launches || (klass != PLT_PROF_ATTN && klass != PLT_PROF_GEMM))
    return fail(PLT_EINVAL, "plt_profile_read: bad argument");
  HIP_TRY(hipStreamSynchronize(m->stream));
  double sum = 0.0; int64_t cnt = 0;
  for (const ProfRec& r : m->prof_used) {
    if (r.klass != klass) continue;
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, r.a, r.b));
    sum += ms; ++cnt;
  }
  *ms_sum = sum; *launches = cnt;
  if (reset) {
    m->prof_free.insert(m->prof_free.end(), m->prof_used.begin(), m->prof_used.end());
    m->prof_used.clear();
  }
  return PLT_OK;
}

// ------------------------------------------------------------------------------ KV layout
// is_clp: the cross-loop-parallel schedule (L rows per sequence in one pass, shift + carry): the
// method itself and its two ablations; only PLT_MODE_CLP has the gated window (rings).
static bool is_clp(const plt_config& c) { return c.mode != PLT_MODE_VANILLA_LOOP; }
static bool is_plt(const plt_config& c) { return c.mode == PLT_MODE_CLP; }
static int n_caches_of(const plt_config& c) {
  return (c.mode == PLT_MODE_CLP || c.mode == PLT_MODE_CLP_SHARE_ONLY) ? 1 : c.n_loops;
}
static int n_rings_of(const plt_config& c) { return is_plt(c) ? c.n_loops - 1 : 0; }
// how one pass of the stack treats K/V and attention
enum { V_PLT = 0,         // loop 1: shared cache; loops >= 2: ring + gated window + shared cache (Alg. 3)
       V_PLAIN = 1,       // every row: plain causal attention over the cache it also appends to
       V_SHARE_ONLY = 2,  // loop 1 appends; loops >= 2 append nothing and attend the shared cache only
       V_OWN_KV = 3 };    // decode rows of loop l append to and attend cache l (one pass, L caches)

extern "C" size_t plt_kv_bytes(const plt_model* m, int32_t batch, int32_t max_ctx) {
  if (!m || batch < 1 || max_ctx < 1) { fail(PLT_EINVAL, "plt_kv_bytes: bad argument"); return 0; }
  const plt_config& c = m->cfg;
  const size_t share = (size_t)batch * c.n_kv_heads * pad_kv(max_ctx, m->kv8) * c.head_dim;
  const size_t ring = (size_t)batch * n_rings_of(c) * c.n_kv_heads * pad_kv(c.window > 0 ? c.window : 1, m->kv8) * c.head_dim;
  const size_t sl = m->phys_layers > 0 && m->phys_layers < c.n_layers ? m->phys_layers : c.n_layers;
  return align256(2 * share * sl * n_caches_of(c) * m->kes) + align256(2 * ring * c.n_layers * m->kes);
}

extern "C" size_t plt_kv_logical_bytes(const plt_model* m, int32_t batch, int32_t n_ctx) {
  if (!m || batch < 1 || n_ctx < 0) { fail(PLT_EINVAL, "plt_kv_logical_bytes: bad argument"); return 0; }
  const plt_config& c = m->cfg;
  const size_t per = (size_t)2 * c.n_layers * c.n_kv_heads * c.head_dim * m->kes * batch;
  if (is_plt(c)) return per * ((size_t)n_ctx + (size_t)(c.n_loops - 1) * c.window);
  return per * (size_t)n_caches_of(c) * n_ctx;
}

static void kv_release(plt_kv* kv) {
  if (!kv) return;
  if (kv->graph_exec) (void)hipGraphExecDestroy(kv->graph_exec);
  void* ptrs[] = {kv->x, kv->a, kv->gout, kv->q, kv->z, kv->y, kv->act, kv->carry, kv->pos_dev, kv->attn_scratch,
                  kv->arg_v, kv->arg_i, kv->moe_idx, kv->a_codes, kv->a_scales, kv->act_sc, kv->dbg_codes, kv->dbg_scales};
  for (void* p : ptrs) if (p) (void)hipFree(p);
  delete kv;
}

extern "C" void plt_kv_free(plt_kv* kv) { kv_release(kv); }

static int mx_max_k(const plt_config& c) {
  int k = c.d_model; if (c.ffn_hidden > k) k = c.ffn_hidden; if (c.n_heads * c.head_dim > k) k = c.n_heads * c.head_dim;
  return k;
}
static size_t gemm_out_need(const plt_config& c, int M, int N, int K, bool head = false) {
  if (c.w_dtype == PLT_MXFP4 && !head) return (size_t)gemm_mx_splits(M, N, K) * M * N;
  const int S = c.dtype == PLT_BF16 ? gemm_bf16_splits_any(M, N, K) : 1;
  return (size_t)S * M * N;
}

extern "C" int plt_kv_alloc(plt_model* m, int32_t batch, int32_t max_ctx, void* dev_buf, size_t nbytes,
                            plt_kv** out) {
  if (!out) return fail(PLT_EINVAL, "plt_kv_alloc: null output pointer");
  *out = nullptr;
  if (!m || batch < 1 || max_ctx < 1 || !dev_buf) return fail(PLT_EINVAL, "plt_kv_alloc: bad argument");
  if (((uintptr_t)dev_buf) & 255) return fail(PLT_EINVAL, "plt_kv_alloc: buffer must be 256-byte aligned");
  const size_t need = plt_kv_bytes(m, batch, max_ctx);
  if (nbytes < need) return fail(PLT_ENOMEM, "plt_kv_alloc: buffer has %zu bytes, layout needs %zu", nbytes, need);
  const plt_config& c = m->cfg;
  if ((long)batch * c.n_loops > 60000) return fail(PLT_EINVAL, "plt_kv_alloc: batch * n_loops too large");
  plt_kv* kv = new (std::nothrow) plt_kv();
  if (!kv) return fail(PLT_ENOMEM, "plt_kv_alloc: out of host memory");
  kv->m = m; kv->B = batch; kv->max_ctx = max_ctx; kv->n_pad = pad_kv(max_ctx, m->kv8);
  kv->w_pad = pad_kv(c.window > 0 ? c.window : 1, m->kv8);
  kv->n_caches = n_caches_of(c); kv->n_rings = n_rings_of(c);
  kv->buf = (char*)dev_buf;
  kv->share_elems = (size_t)batch * c.n_kv_heads * kv->n_pad * c.head_dim;
  kv->ring_elems = (size_t)batch * kv->n_rings * c.n_kv_heads * kv->w_pad * c.head_dim;
  kv->share_layers = m->phys_layers > 0 && m->phys_layers < c.n_layers ? m->phys_layers : c.n_layers;
  kv->ring_base = align256(2 * kv->share_elems * kv->share_layers * kv->n_caches * m->kes);
  kv->pos = 0; kv->started = false;
  // cleared so that padded / not-yet-written slots hold finite values (masked keys multiply
  // their value rows by zero weights, which must not meet NaN bit patterns)
  hipError_t e = hipMemsetAsync(dev_buf, 0, need, m->stream);
  const int L = c.n_loops, R = is_clp(c) ? batch * L : batch;
  const int d = c.d_model, Hq = c.n_heads, Hkv = c.n_kv_heads, D = c.head_dim, F = c.ffn_hidden, V = c.vocab;
  const int Nqkv = (Hq + 2 * Hkv) * D;
  size_t go = gemm_out_need(c, R, Nqkv, d);
  size_t t;
  if ((t = gemm_out_need(c, R, d, Hq * D)) > go) go = t;
  if (c.n_experts > 0) {
    if ((t = (size_t)c.top_k * R * d) > go) go = t;                  // one output slab per selected expert
  } else {
    if ((t = gemm_out_need(c, R, 2 * F, d)) > go) go = t;
    if ((t = gemm_out_need(c, R, d, F)) > go) go = t;
  }
  if ((t = gemm_out_need(c, batch, V, d, true)) > go) go = t;
  kv->gout_elems = go;
  kv->attn_scratch_bytes = attn_mfma_scratch_bytes(batch, is_clp(c) ? L : 1, Hq, Hkv, D, attn_mfma_max_default_splits(batch, Hkv));
  auto dmalloc = [&](void** p, size_t bytes) { if (e == hipSuccess) e = hipMalloc(p, bytes ? bytes : 256); };
  dmalloc((void**)&kv->x, (size_t)R * d * 4);
  dmalloc(&kv->a, (size_t)R * d * (m->mx ? 4 : m->es));
  dmalloc((void**)&kv->gout, go * 4);
  dmalloc(&kv->q, (size_t)R * Hq * D * m->es);
  dmalloc((void**)&kv->z, (size_t)R * Hq * 4);
  dmalloc(&kv->y, (size_t)R * Hq * D * m->es);
  dmalloc(&kv->act, (size_t)R * (c.n_experts > 0 ? c.top_k : 1) * F * (m->mx ? 4 : m->es));
  if (m->mx) {
    const int maxK = mx_max_k(c);
    dmalloc((void**)&kv->a_codes, (size_t)R * maxK);
    dmalloc((void**)&kv->a_scales, (size_t)R * mx_ascale_row_bytes(maxK));
    if (c.n_experts > 0) {
      const size_t nb = (size_t)R * c.top_k * mx_ascale_row_bytes(F);
      dmalloc((void**)&kv->act_sc, nb);
      if (e == hipSuccess) e = hipMemsetAsync(kv->act_sc, 0, nb, m->stream);     // pad bytes stay 0
    }
  }
  if (c.n_experts > 0) dmalloc(&kv->moe_idx, moe_index_bytes(R, c.top_k, c.n_experts));
  dmalloc((void**)&kv->carry, (size_t)batch * (L > 1 ? L - 1 : 1) * d * 4);
  dmalloc((void**)&kv->pos_dev, (size_t)batch * 4);
  dmalloc(&kv->attn_scratch, kv->attn_scratch_bytes);
  dmalloc((void**)&kv->arg_v, (size_t)argmax_scratch_elems(batch) * 4);
  dmalloc((void**)&kv->arg_i, (size_t)argmax_scratch_elems(batch) * 4);
  if (e == hipSuccess) e = hipMemsetAsync(kv->attn_scratch, 0, kv->attn_scratch_bytes, m->stream);
  if (e == hipSuccess) e = hipMemsetAsync(kv->carry, 0, (size_t)batch * (L > 1 ? L - 1 : 1) * d * 4, m->stream);
  if (e == hipSuccess) e = hipMemsetAsync(kv->x, 0, (size_t)R * d * 4, m->stream);
  if (e != hipSuccess) {
    kv_release(kv);
    return fail(e == hipErrorOutOfMemory ? PLT_ENOMEM : PLT_EHIP, "plt_kv_alloc: %s", hipGetErrorString(e));
  }
  *out = kv;
  return PLT_OK;
}

extern "C" int plt_kv_alias_layers(plt_model* m, int32_t phys_layers) {
  if (!m || phys_layers < 0) return fail(PLT_EINVAL, "plt_kv_alias_layers: bad argument");
  m->phys_layers = phys_layers;
  return PLT_OK;
}

extern "C" int32_t plt_kv_position(const plt_kv* kv) {
  if (!kv) return fail(PLT_EINVAL, "plt_kv_position: null kv");
  return kv->pos;
}

static KvView kv_view(const plt_kv* kv, int layer, int cache) {
  const plt_model* m = kv->m;
  const plt_config& c = m->cfg;
  KvView v;
  const size_t es = m->kes;
  char* sb = kv->buf + ((size_t)cache * kv->share_layers + layer % kv->share_layers) * 2 * kv->share_elems * es;
  v.k_share = sb; v.v_share = sb + kv->share_elems * es;
  if (kv->n_rings > 0) {
    char* rb = kv->buf + kv->ring_base + (size_t)layer * 2 * kv->ring_elems * es;
    v.k_ring = rb; v.v_ring = rb + kv->ring_elems * es;
  } else { v.k_ring = nullptr; v.v_ring = nullptr; }
  v.k_loc = nullptr; v.v_loc = nullptr;
  v.n_pad = kv->n_pad; v.w_pad = kv->w_pad; v.n_pad_loc = 0;
  v.w = c.window > 0 ? c.window : 1; v.n_rings = kv->n_rings; v.b0 = 0;
  v.cache_stride = (size_t)kv->share_layers * 2 * kv->share_elems;   // elements between cache c and c + 1 of one layer
  return v;
}

// ------------------------------------------------------------------------------ scheduler
struct Work {            // activation buffers one pass of the stack runs on
  float* x; void* a; float* gout; void* q; float* z; void* y; void* act;
  float* attn_tmp;   // prefill only: float [rows, Hq*D]
  void* moe_idx;     // mixture-of-experts models: routing lists (moe_index_bytes for the pass's rows)
  uint8_t *a_codes, *a_scales;   // low-bit models: e4m3 codes / block scales of the next projection's input
  uint8_t* act_sc;               // low-bit mixture-of-experts models: block scales of the experts' hidden rows
};

static int run_gemm(plt_model* m, const void* a, const void* w, float* out, int M, int N, int K,
                    bool decode = false) {
  ProfScope prof(m, PLT_PROF_GEMM, decode);
  if (m->cfg.dtype == PLT_BF16) {
    launch_gemm_bf16_any(m->stream, (const bf16_t*)a, (const bf16_t*)w, out, M, N, K);
    return gemm_bf16_splits_any(M, N, K);
  }
  launch_gemm_f32(m->stream, (const float*)a, (const float*)w, out, M, N, K);
  return 1;
}

// x += sum of the GEMM slabs; a = RMSNorm(x) * gain as the next projection's input: the model dtype, or (low-bit
// models) float rows quantised to e4m3 blocks
template <typename T>
static void norm_to_a(plt_model* m, const Work& wk, const float* partials, int S, size_t slab, const float* gain, int R) {
  const plt_config& c = m->cfg;
  if (m->mx && gain && resid_norm_mx_applies(c.d_model) && (slab & 3) == 0) {
    launch_resid_norm_mx(m->stream, wk.x, partials, S, slab, gain, c.norm_eps, wk.a_codes, wk.a_scales, R, c.d_model);
  } else if (m->mx && gain) {
    launch_resid_norm<float>(m->stream, wk.x, 1, 0, partials, S, slab, gain, c.norm_eps, (float*)wk.a, R, c.d_model);
    launch_mx_quant_a<float>(m->stream, (const float*)wk.a, wk.a_codes, wk.a_scales, R, c.d_model);
  } else {
    launch_resid_norm<T>(m->stream, wk.x, 1, 0, partials, S, slab, gain, c.norm_eps, gain ? (T*)wk.a : (T*)nullptr, R, c.d_model);
  }
}
static int run_gemm_mx(plt_model* m, const Work& wk, const void* w, const uint8_t* w_sc, int M, int N, int K, bool decode) {
  ProfScope prof(m, PLT_PROF_GEMM, decode);
  launch_gemm_mx(m->stream, wk.a_codes, wk.a_scales, (const uint8_t*)w, w_sc, wk.gout, M, N, K);
  return gemm_mx_splits(M, N, K);
}

// test hook: keeps a copy of the quantised input of projection `slot` (0 QKV, 1 output, 2 gate/up, 3 down)
static void dbg_capture(plt_model* m, plt_kv* kv, const Work& wk, int slot, int R, int K) {
  if (!kv->dbg_on) return;
  (void)hipMemcpyAsync(kv->dbg_codes + slot * kv->dbg_codes_slot, wk.a_codes, (size_t)R * K, hipMemcpyDeviceToDevice, m->stream);
  (void)hipMemcpyAsync(kv->dbg_scales + slot * kv->dbg_scales_slot, wk.a_scales, (size_t)R * mx_ascale_row_bytes(K),
                       hipMemcpyDeviceToDevice, m->stream);
}

template <typename T>
static void stack_pass(plt_model* m, plt_kv* kv, const Work& wk, int R, RowMap rm, int cache, int variant,
                       KvView loc /*prefill local K/V + b0*/, int Bc, int n_prefill, int attn_L,
                       const float* next_gain /*norm applied after the last layer, or null*/,
                       int layer_beg = 0, int layer_end = -1 /* -1: all layers */) {
  // Runs layers layer_beg .. layer_end - 1 of block f on the R rows in wk.x (a = RMSNorm(x) with the first of these
  // layers' gain is already in wk.a).
  const plt_config& c = m->cfg;
  hipStream_t s = m->stream;
  const int d = c.d_model, Hq = c.n_heads, Hkv = c.n_kv_heads, D = c.head_dim, F = c.ffn_hidden;
  const int Nqkv = (Hq + 2 * Hkv) * D;
  Dims dm{rm.prefill ? Bc : kv->B, attn_L, Hq, Hkv, D, d, F, c.vocab};
  if (layer_end < 0) layer_end = c.n_layers;
  const bool big_resid = c.dtype == PLT_BF16 && !m->mx;
  for (int l = layer_beg; l < layer_end; ++l) {
    const LayerW& w = m->layers[l];
    KvView v = kv_view(kv, l, cache);
    v.k_loc = loc.k_loc; v.v_loc = loc.v_loc; v.n_pad_loc = loc.n_pad_loc; v.b0 = loc.b0;
    if (m->mx) dbg_capture(m, kv, wk, 0, R, d);
    int S = 1;
    if (!m->mx && c.dtype == PLT_BF16 && rm.prefill && variant != V_OWN_KV && R % rm.rows_per_seq == 0 &&
        gemm_rope_applies(R, Nqkv, d, D)) {
      // prefill chunk: S3 runs as the projection's epilogue (no float QKV matrix)                  // Alg. 3 l.1, l.4
      ProfScope prof(m, PLT_PROF_GEMM, false);
      launch_gemm_big_rope(s, (const bf16_t*)wk.a, (const bf16_t*)w.wqkv, R, Nqkv, d, w.gate_w, w.gate_b, (bf16_t*)wk.q,
                           wk.z, v, rm.rows_per_seq, rm.loop_fixed, dm, m->inv_freq, variant, m->kv8);
    } else if (!m->mx && c.dtype == PLT_BF16 && !rm.prefill && gemm_rope_rows_applies(R, Nqkv, d, D)) {
      // decode rows: likewise (row (b, l) at position pos[b])                                      // Alg. 1 l.5-7
      ProfScope prof(m, PLT_PROF_GEMM, true);
      launch_gemm_rope_rows(s, (const bf16_t*)wk.a, (const bf16_t*)w.wqkv, R, Nqkv, d, w.gate_w, w.gate_b, (bf16_t*)wk.q,
                            wk.z, v, rm.pos, rm.rows_per_seq, dm, m->inv_freq, variant, m->kv8);
    } else if (m->mx && c.dtype == PLT_BF16 && !rm.prefill && gemm_mx_rope_rows_applies(R, Nqkv, d, D)) {
      // low-bit decode rows: likewise
      ProfScope prof(m, PLT_PROF_GEMM, true);
      launch_gemm_mx_rope_rows(s, wk.a_codes, wk.a_scales, (const uint8_t*)w.wqkv, w.wqkv_sc, R, Nqkv, d, w.gate_w, w.gate_b,
                               (bf16_t*)wk.q, wk.z, v, rm.pos, rm.rows_per_seq, dm, m->inv_freq, variant, m->kv8);
    } else {
      S = m->mx ? run_gemm_mx(m, wk, w.wqkv, w.wqkv_sc, R, Nqkv, d, !rm.prefill)
                : run_gemm(m, wk.a, w.wqkv, wk.gout, R, Nqkv, d, !rm.prefill);                         // Alg. 3 l.1
      if (m->kv8)
        launch_rope_append<bf16_t, fp8_t>(s, wk.gout, S, (size_t)R * Nqkv, w.gate_w, w.gate_b, (bf16_t*)wk.q, wk.z, v, rm,
                                          R, dm, m->inv_freq, variant);
      else
        launch_rope_append<T, T>(s, wk.gout, S, (size_t)R * Nqkv, w.gate_w, w.gate_b, (T*)wk.q, wk.z, v, rm, R,
                                 dm, m->inv_freq, variant);
    }
    const bool dec = !rm.prefill;
    const int plain = variant != V_PLT;
    // low-bit models, decode: the attention kernel writes y as e4m3 blocks itself (no scale padding needed)
    const bool y_mx = m->mx && dec && ((Hq * D) % 512) == 0;
    uint8_t* yc = y_mx ? wk.a_codes : nullptr;
    uint8_t* ysc = y_mx ? wk.a_scales : nullptr;
    if (c.dtype == PLT_BF16) {                                                              // Alg. 3 l.2-5
      ProfScope prof(m, PLT_PROF_ATTN, dec);
      if (rm.prefill) {
        launch_attn_prefill_mfma(s, (const bf16_t*)wk.q, wk.z, (bf16_t*)wk.y, wk.attn_tmp, v, Bc, n_prefill,
                                 rm.loop_fixed, dm, plain ? 1 : 0, m->kv8);
      } else {
        const int G = Hq / Hkv;
        if (variant == V_OWN_KV) {
          // loop l's rows attend cache l: one launch per loop, G rows per (sequence, kv head) stream
          Dims d1 = dm; d1.L = 1;
          const int ns = attn_mfma_default_splits(kv->B, Hkv, 1, G, kv->pos + 1, m->kv8);
          for (int lp = 0; lp < attn_L; ++lp) {
            KvView vl = v;
            vl.k_share = (char*)v.k_share + (size_t)lp * v.cache_stride * m->kes;
            vl.v_share = (char*)v.v_share + (size_t)lp * v.cache_stride * m->kes;
            launch_attn_decode_mfma(s, (const bf16_t*)wk.q, wk.z, (bf16_t*)wk.y, vl, kv->pos_dev, 0, 0, d1, 1,
                                    kv->attn_scratch, ns, lp, attn_L, m->kv8, attn_mfma_max_default_splits(kv->B, Hkv), yc, ysc);
          }
        } else {
          const int ns = attn_mfma_default_splits(kv->B, Hkv, attn_L, G, kv->pos + 1, m->kv8);
          launch_attn_decode_mfma(s, (const bf16_t*)wk.q, wk.z, (bf16_t*)wk.y, v, kv->pos_dev, 0, 0, dm,
                                  plain ? 1 : 0, kv->attn_scratch, ns, 0, 0, m->kv8, attn_mfma_max_default_splits(kv->B, Hkv),
                                  yc, ysc);
        }
      }
    } else {
      ProfScope prof(m, PLT_PROF_ATTN, dec);
      launch_attn_f32(s, (const float*)wk.q, wk.z, (float*)wk.y, v, rm, R, dm, variant == V_OWN_KV && dec ? 3 : plain);
    }
    if (m->mx) {                                                                                 // Alg. 3 l.6
      if (!y_mx) launch_mx_quant_a<bf16_t>(s, (const bf16_t*)wk.y, wk.a_codes, wk.a_scales, R, Hq * D);
      dbg_capture(m, kv, wk, 1, R, Hq * D);
      S = run_gemm_mx(m, wk, w.wo, w.wo_sc, R, d, Hq * D, dec);
    } else if (big_resid && gemm_big_applies(R, d, Hq * D)) {      // many rows: the residual add is the projection's epilogue
      ProfScope prof(m, PLT_PROF_GEMM, dec);
      launch_gemm_big_resid(s, (const bf16_t*)wk.y, (const bf16_t*)w.wo, wk.x, R, d, Hq * D);
      S = 0;
    } else {
      S = run_gemm(m, wk.y, w.wo, wk.gout, R, d, Hq * D, dec);
    }
    norm_to_a<T>(m, wk, wk.gout, S, (size_t)R * d, w.norm2, R);
    if (m->mx) dbg_capture(m, kv, wk, 2, R, d);
    if (m->mx && c.n_experts > 0) {                          // mixture of experts on low-bit operands
      ProfScope prof(m, PLT_PROF_GEMM, dec);
      launch_moe_ffn_mx(s, wk.a_codes, wk.a_scales, (const bf16_t*)w.router, (const uint8_t*)w.wgu, w.wgu_sc,
                        (const uint8_t*)w.wdown, w.wdown_sc, (uint8_t*)wk.act, wk.act_sc, wk.gout,
                        moe_index_carve(wk.moe_idx, R, c.top_k, c.n_experts), R, d, F, c.n_experts, c.top_k);
      S = c.top_k;
    } else if (m->mx) {                                      // low-bit gate/up and down projections
      if (gemm_mx_swiglu_rows_applies(R, F, d)) {
        // decode rows: SwiGLU + e4m3 blocks in the product's epilogue.  The hidden codes and their scale bytes go to
        // the (otherwise unused, 4 bytes per element) hidden-row buffer: the product's own operand stays intact
        Work wh = wk;
        wh.a_codes = (uint8_t*)wk.act; wh.a_scales = (uint8_t*)wk.act + align256((size_t)R * F);
        {
          ProfScope prof(m, PLT_PROF_GEMM, dec);
          launch_gemm_mx_swiglu_rows(s, wk.a_codes, wk.a_scales, (const uint8_t*)w.wgu, w.wgu_sc, wh.a_codes, wh.a_scales, R, F, d);
        }
        dbg_capture(m, kv, wh, 3, R, F);
        S = run_gemm_mx(m, wh, w.wdown, w.wdown_sc, R, d, F, dec);
      } else {
        S = run_gemm_mx(m, wk, w.wgu, w.wgu_sc, R, 2 * F, d, dec);
        launch_silu_mul_mx(s, wk.gout, S, (size_t)R * 2 * F, wk.a_codes, wk.a_scales, R, F);      // SwiGLU + e4m3 blocks
        dbg_capture(m, kv, wk, 3, R, F);
        S = run_gemm_mx(m, wk, w.wdown, w.wdown_sc, R, d, F, dec);
      }
    } else if (c.n_experts > 0) {                                   // mixture of experts: k slabs, one per selected expert
      ProfScope prof(m, PLT_PROF_GEMM, dec);
      launch_moe_ffn<T>(s, (const T*)wk.a, (const T*)w.router, (const T*)w.wgu, (const T*)w.wdown, (T*)wk.act, wk.gout,
                        moe_index_carve(wk.moe_idx, R, c.top_k, c.n_experts), R, d, F, c.n_experts, c.top_k);
      S = c.top_k;
    } else if (c.dtype == PLT_BF16 && gemm_big_applies(R, 2 * F, d)) {      // many rows: SwiGLU fused into the GEMM epilogue
      launch_gemm_big_swiglu(s, (const bf16_t*)wk.a, (const bf16_t*)w.wgu, (bf16_t*)wk.act, R, F, d);
    } else if (c.dtype == PLT_BF16 && gemm_swiglu_rows_applies(R, F, d)) {   // decode rows: likewise, one tile of rows
      ProfScope prof(m, PLT_PROF_GEMM, dec);
      launch_gemm_swiglu_rows(s, (const bf16_t*)wk.a, (const bf16_t*)w.wgu, (bf16_t*)wk.act, R, F, d);
    } else {
      S = run_gemm(m, wk.a, w.wgu, wk.gout, R, 2 * F, d, dec);
      launch_silu_mul<T>(s, wk.gout, S, (size_t)R * 2 * F, (T*)wk.act, R, F);
    }
    if (c.n_experts == 0 && !m->mx) {
      if (big_resid && gemm_big_applies(R, d, F)) {
        ProfScope prof(m, PLT_PROF_GEMM, dec);
        launch_gemm_big_resid(s, (const bf16_t*)wk.act, (const bf16_t*)w.wdown, wk.x, R, d, F);
        S = 0;
      } else {
        S = run_gemm(m, wk.act, w.wdown, wk.gout, R, d, F, dec);
      }
    }
    const float* gain = l + 1 < c.n_layers ? m->layers[l + 1].norm1 : next_gain;
    if (S > 0 || gain) norm_to_a<T>(m, wk, wk.gout, S, (size_t)R * d, gain, R);      // (nothing left to do otherwise)
  }
}

template <typename T>
static void head_and_argmax(plt_model* m, plt_kv* kv, const Work& wk, int rows, int row_stride, int row_off,
                            int32_t* dev_next, float* dev_logits, bool decode = false) {
  const plt_config& c = m->cfg;
  launch_resid_norm<T>(m->stream, wk.x, row_stride, row_off, nullptr, 0, 0, m->norm_f, c.norm_eps, (T*)wk.a,
                       rows, c.d_model);
  const int S = run_gemm(m, wk.a, m->head, wk.gout, rows, c.vocab, c.d_model, decode);
  launch_argmax(m->stream, wk.gout, S, (size_t)rows * c.vocab, dev_logits, dev_next, rows, c.vocab, kv->arg_v, kv->arg_i);
}

template <typename T>
static int decode_step_t(plt_model* m, plt_kv* kv, const int32_t* dev_tokens, int32_t* dev_next,
                         float* dev_logits) {
  const plt_config& c = m->cfg;
  hipStream_t s = m->stream;
  const int B = kv->B, L = c.n_loops, d = c.d_model;
  Work wk{kv->x, kv->a, kv->gout, kv->q, kv->z, kv->y, kv->act, nullptr, kv->moe_idx, kv->a_codes, kv->a_scales, kv->act_sc};
  KvView none{}; none.b0 = 0;
  if (is_clp(c)) {
    // Alg. 1 l.5-7: rows B_0 = e, B_l = e + H^l[p-1]; the L rows of a sequence run as one pass
    const int R = B * L;
    RowMap rm{0, L, 0, kv->pos_dev};
    launch_embed<T>(s, dev_tokens, (const T*)m->emb, kv->carry, nullptr, kv->x, R, d, rm, L, 1, c.vocab);
    norm_to_a<T>(m, wk, nullptr, 0, 0, m->layers[0].norm1, R);
    const int variant = c.mode == PLT_MODE_CLP ? V_PLT : (c.mode == PLT_MODE_CLP_SHARE_ONLY ? V_SHARE_ONLY : V_OWN_KV);
    stack_pass<T>(m, kv, wk, R, rm, 0, variant, none, 0, 0, L, nullptr);
    launch_carry_update(s, kv->x, kv->carry, B, L, d);
    head_and_argmax<T>(m, kv, wk, B, L, L - 1, dev_next, dev_logits, true);                       // Alg. 1 l.8-9
  } else {
    // Eq. (1): L serial passes of B rows, loop l on its own cache l
    RowMap rm{0, 1, 0, kv->pos_dev};
    launch_embed<T>(s, dev_tokens, (const T*)m->emb, nullptr, nullptr, kv->x, B, d, rm, 1, 0, c.vocab);
    norm_to_a<T>(m, wk, nullptr, 0, 0, m->layers[0].norm1, B);
    for (int l = 0; l < L; ++l)
      stack_pass<T>(m, kv, wk, B, rm, l, V_PLAIN, none, 0, 0, 1, l + 1 < L ? m->layers[0].norm1 : nullptr);
    head_and_argmax<T>(m, kv, wk, B, 1, 0, dev_next, dev_logits, true);
  }
  launch_pos_set(s, kv->pos_dev, B, 1, 1);
  return PLT_OK;
}

// The one launch parameter of a decode step that the HOST derives from the position (everything else the kernels
// read from the device-side position counter): the number of workgroups a stream of the attention is split over.
static int step_splits(const plt_model* m, const plt_kv* kv) {
  const plt_config& c = m->cfg;
  if (c.dtype != PLT_BF16) return 0;
  const int G = c.n_heads / c.n_kv_heads;
  const int L = (is_clp(c) && c.mode != PLT_MODE_CLP_OWN_KV) ? c.n_loops : 1;
  return attn_mfma_default_splits(kv->B, c.n_kv_heads, L, G, kv->pos + 1, m->kv8);
}

// Replays the step as a HIP graph: captured (stream capture of the very launch sequence the eager step issues) the
// first time and whenever the arguments or the attention split count change, replayed otherwise.  No memset nodes:
// the step clears nothing.  A failed capture or instantiation launches nothing and is reported.
static int decode_step_graph(plt_model* m, plt_kv* kv, const int32_t* dev_tokens, int32_t* dev_next, float* dev_logits) {
  const int splits = step_splits(m, kv);
  if (!kv->graph_exec || kv->g_tokens != dev_tokens || kv->g_next != dev_next || kv->g_logits != dev_logits || kv->g_splits != splits) {
    if (kv->graph_exec) { (void)hipGraphExecDestroy(kv->graph_exec); kv->graph_exec = nullptr; }
    hipGraph_t graph = nullptr;
    if (m->stream == nullptr) return fail(PLT_EHIP, "plt_decode_step: graph replay needs a stream of its own (the model was created on the NULL stream)");
    hipError_t e = hipStreamBeginCapture(m->stream, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) { (void)hipGetLastError(); return fail(PLT_EHIP, "plt_decode_step: hipStreamBeginCapture: %s", hipGetErrorString(e)); }
    const int rc = m->cfg.dtype == PLT_BF16 ? decode_step_t<bf16_t>(m, kv, dev_tokens, dev_next, dev_logits)
                                            : decode_step_t<float>(m, kv, dev_tokens, dev_next, dev_logits);
    e = hipStreamEndCapture(m->stream, &graph);            // always ends the capture, also after a failed launch
    if (rc != PLT_OK || e != hipSuccess || !graph) {
      if (graph) (void)hipGraphDestroy(graph);
      (void)hipGetLastError();
      return fail(PLT_EHIP, "plt_decode_step: stream capture failed: %s", hipGetErrorString(e));
    }
    e = hipGraphInstantiate(&kv->graph_exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e != hipSuccess) { kv->graph_exec = nullptr; return fail(PLT_EHIP, "plt_decode_step: hipGraphInstantiate: %s", hipGetErrorString(e)); }
    kv->g_tokens = dev_tokens; kv->g_next = dev_next; kv->g_logits = dev_logits; kv->g_splits = splits;
  }
  HIP_TRY(hipGraphLaunch(kv->graph_exec, m->stream));
  return PLT_OK;
}

extern "C" int plt_use_graph(plt_model* m, int32_t on) {
  if (!m) return fail(PLT_EINVAL, "plt_use_graph: null model");
  m->use_graph = on != 0;
  return PLT_OK;
}

extern "C" int plt_decode_step(plt_model* m, plt_kv* kv, const int32_t* dev_tokens, int32_t* dev_next,
                               float* dev_logits) {
  if (!m || !kv || kv->m != m || !dev_tokens || !dev_next) return fail(PLT_EINVAL, "plt_decode_step: bad argument");
  if (!kv->started) return fail(PLT_ESTATE, "plt_decode_step: plt_prefill (or plt_kv_set_position) must come first");
  if (kv->pos >= kv->max_ctx) return fail(PLT_ECTXFULL, "plt_decode_step: context full (%d positions)", kv->max_ctx);
  if (m->use_graph && m->profile == 0) {       // (the event instrumentation records events: eager only)
    // a capture or instantiation that fails has launched nothing: the error is reported and the state is unchanged
    const int rc = decode_step_graph(m, kv, dev_tokens, dev_next, dev_logits);
    if (rc == PLT_OK) kv->pos += 1;
    return rc;
  }
  int rc = m->cfg.dtype == PLT_BF16 ? decode_step_t<bf16_t>(m, kv, dev_tokens, dev_next, dev_logits)
                                    : decode_step_t<float>(m, kv, dev_tokens, dev_next, dev_logits);
  if (rc == PLT_OK && hipGetLastError() != hipSuccess) rc = fail(PLT_EHIP, "plt_decode_step: a kernel launch failed");
  if (rc != PLT_OK) {
    // some launches may have run (device-side position counter included): the host and device views of the
    // position can no longer be trusted, so the object asks for plt_prefill / plt_kv_set_position again
    kv->started = false;
    return rc;
  }
  kv->pos += 1;
  return PLT_OK;
}

// ------------------------------------------------------------------------------ prefill
static const int PREFILL_ROWS = 16384;   // activation rows per chunk of whole sequences

// Layout of the prefill workspace: one chunk's activation buffers, carved from one caller buffer.
struct PrefillPlan {
  int Bc, Rc, n_pad_loc;
  size_t o_x, o_h, o_a, o_g, o_q, o_z, o_y, o_act, o_ac, o_as, o_hs, o_moe, o_kl, o_vl, o_tmp, total;
  size_t kv_loc_bytes, hs_bytes;
};
static PrefillPlan prefill_plan(const plt_model* m, const plt_kv* kv, int n) {
  const plt_config& c = m->cfg;
  const int B = kv->B, L = c.n_loops, d = c.d_model, Hq = c.n_heads, Hkv = c.n_kv_heads, D = c.head_dim,
            F = c.ffn_hidden, V = c.vocab, es = m->es, kes = m->kes;
  const int Nqkv = (Hq + 2 * Hkv) * D;
  PrefillPlan p;
  p.Bc = PREFILL_ROWS / n; if (p.Bc < 1) p.Bc = 1; if (p.Bc > B) p.Bc = B;
  p.Rc = p.Bc * n;
  p.n_pad_loc = pad_kv(n, m->kv8);
  const int Rc = p.Rc, Bc = p.Bc;
  size_t go = gemm_out_need(c, Rc, Nqkv, d), t;
  if ((t = gemm_out_need(c, Rc, d, Hq * D)) > go) go = t;
  const int E = c.n_experts, topk = E > 0 ? c.top_k : 1;
  if (E > 0) {
    if ((t = (size_t)topk * Rc * d) > go) go = t;
  } else {
    if ((t = gemm_out_need(c, Rc, 2 * F, d)) > go) go = t;
    if ((t = gemm_out_need(c, Rc, d, F)) > go) go = t;
  }
  if ((t = gemm_out_need(c, Bc, V, d, true)) > go) go = t;
  size_t off = 0;
  auto carve = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
  const size_t wes = m->mx ? 4 : es;      // low-bit models keep projection inputs as float until they are quantised
  p.kv_loc_bytes = (size_t)Bc * Hkv * p.n_pad_loc * D * kes;
  p.hs_bytes = m->mx && E > 0 ? (size_t)Rc * topk * mx_ascale_row_bytes(F) : 0;
  p.o_x = carve((size_t)Rc * d * 4); p.o_h = carve((size_t)Rc * d * 4); p.o_a = carve((size_t)Rc * d * wes);
  p.o_g = carve(go * 4); p.o_q = carve((size_t)Rc * Hq * D * es); p.o_z = carve((size_t)Rc * Hq * 4);
  p.o_y = carve((size_t)Rc * Hq * D * es); p.o_act = carve((size_t)Rc * topk * F * wes);
  p.o_ac = carve(m->mx ? (size_t)Rc * mx_max_k(c) : 256);
  p.o_as = carve(m->mx ? (size_t)Rc * mx_ascale_row_bytes(mx_max_k(c)) : 256);
  p.o_hs = carve(p.hs_bytes ? p.hs_bytes : 256);
  p.o_moe = carve(E > 0 ? moe_index_bytes(Rc, topk, E) : 256);
  p.o_kl = carve(p.kv_loc_bytes); p.o_vl = carve(p.kv_loc_bytes);
  p.o_tmp = carve((L > 1 && is_plt(c) && es == 2) ? (size_t)Rc * Hq * D * 4 : 256);
  p.total = off;
  return p;
}

template <typename T>
static int prefill_t(plt_model* m, plt_kv* kv, const int32_t* dev_tokens, int n, int32_t* dev_next,
                     float* dev_logits, char* ws) {
  const plt_config& c = m->cfg;
  hipStream_t s = m->stream;
  const int B = kv->B, L = c.n_loops, d = c.d_model, V = c.vocab;
  const PrefillPlan pl = prefill_plan(m, kv, n);
  const int Bc = pl.Bc;
  // the chunk's own-loop K/V (and, low-bit mixture-of-experts models, the pad bytes of the hidden rows' scales) start
  // from zero; cleared by a fill kernel, not a memset node, so that the call may be captured in a HIP graph
  launch_fill_zero(s, ws + pl.o_kl, pl.o_vl + pl.kv_loc_bytes - pl.o_kl);
  if (pl.hs_bytes) launch_fill_zero(s, ws + pl.o_hs, pl.hs_bytes);
  Work wk{(float*)(ws + pl.o_x), ws + pl.o_a, (float*)(ws + pl.o_g), ws + pl.o_q, (float*)(ws + pl.o_z), ws + pl.o_y,
          ws + pl.o_act, (float*)(ws + pl.o_tmp), ws + pl.o_moe, (uint8_t*)(ws + pl.o_ac), (uint8_t*)(ws + pl.o_as),
          (uint8_t*)(ws + pl.o_hs)};
  float* hprev = (float*)(ws + pl.o_h);
  for (int b0 = 0; b0 < B; b0 += Bc) {
    const int bc = b0 + Bc <= B ? Bc : B - b0;
    const int R = bc * n;
    const int32_t* toks = dev_tokens + (size_t)b0 * n;
    KvView loc{}; loc.k_loc = ws + pl.o_kl; loc.v_loc = ws + pl.o_vl; loc.n_pad_loc = pl.n_pad_loc; loc.b0 = b0;
    for (int l = 0; l < L; ++l) {
      RowMap rm{1, n, is_clp(c) ? l : 0, nullptr};
      if (is_clp(c)) {
        // Alg. 2 l.1-2 (l = 0) and l.4-6 (l >= 1): B = E + shift_right(H^(l))
        launch_embed<T>(s, toks, (const T*)m->emb, nullptr, hprev, wk.x, R, d, rm, L, 1, c.vocab);
        norm_to_a<T>(m, wk, nullptr, 0, 0, m->layers[0].norm1, R);
        // own-KV ablation: loop l is a plain pass over its own cache l; share-only: loops >= 2 append nothing
        const int variant = c.mode == PLT_MODE_CLP ? V_PLT : (c.mode == PLT_MODE_CLP_SHARE_ONLY ? V_SHARE_ONLY : V_PLAIN);
        stack_pass<T>(m, kv, wk, R, rm, c.mode == PLT_MODE_CLP_OWN_KV ? l : 0, variant, loc, bc, n, L, nullptr);
        if (l + 1 < L) {
          launch_prefill_carry(s, wk.x, kv->carry, b0, bc, n, L, l, d);
          launch_shift_copy(s, wk.x, hprev, (size_t)R * d);
        }
      } else {
        if (l == 0) {
          launch_embed<T>(s, toks, (const T*)m->emb, nullptr, nullptr, wk.x, R, d, rm, 1, 0, c.vocab);
          norm_to_a<T>(m, wk, nullptr, 0, 0, m->layers[0].norm1, R);
        }
        stack_pass<T>(m, kv, wk, R, rm, l, V_PLAIN, loc, bc, n, 1, l + 1 < L ? m->layers[0].norm1 : nullptr);
      }
    }
    head_and_argmax<T>(m, kv, wk, bc, n, n - 1, dev_next + b0, dev_logits ? dev_logits + (size_t)b0 * V : nullptr);
  }
  launch_pos_set(s, kv->pos_dev, B, n, 0);
  return PLT_OK;
}

static int prefill_check(const plt_model* m, const plt_kv* kv, int32_t n, const char* who) {
  if (!m || !kv || kv->m != m) return fail(PLT_EINVAL, "%s: bad model / kv object", who);
  if (n < 1) return fail(PLT_EINVAL, "%s: empty prompt", who);
  if (n > kv->max_ctx) return fail(PLT_ECTXFULL, "%s: prompt of %d exceeds max_ctx %d", who, n, kv->max_ctx);
  int Bc = PREFILL_ROWS / n; if (Bc < 1) Bc = 1; if (Bc > kv->B) Bc = kv->B;
  if ((long)Bc * n > 60000) return fail(PLT_EINVAL, "%s: prompt too long (%d positions; limit 60000)", who, n);
  return PLT_OK;
}

extern "C" size_t plt_prefill_workspace_bytes(const plt_model* m, const plt_kv* kv, int32_t n) {
  if (prefill_check(m, kv, n, "plt_prefill_workspace_bytes") != PLT_OK) return 0;
  return prefill_plan(m, kv, n).total;
}

extern "C" int plt_prefill(plt_model* m, plt_kv* kv, const int32_t* dev_tokens, int32_t n, int32_t* dev_next,
                           float* dev_logits, void* dev_workspace, size_t workspace_bytes) {
  if (!dev_tokens || !dev_next) return fail(PLT_EINVAL, "plt_prefill: null tokens / next pointer");
  int rc = prefill_check(m, kv, n, "plt_prefill");
  if (rc != PLT_OK) return rc;
  const size_t need = prefill_plan(m, kv, n).total;
  if (!dev_workspace || (((uintptr_t)dev_workspace) & 255)) return fail(PLT_EINVAL, "plt_prefill: workspace must be a 256-byte aligned device buffer");
  if (workspace_bytes < need) return fail(PLT_ENOMEM, "plt_prefill: workspace has %zu bytes, this prompt needs %zu", workspace_bytes, need);
  kv->started = false;              // a failure below leaves the object in need of a new prefill
  rc = m->cfg.dtype == PLT_BF16 ? prefill_t<bf16_t>(m, kv, dev_tokens, n, dev_next, dev_logits, (char*)dev_workspace)
                                : prefill_t<float>(m, kv, dev_tokens, n, dev_next, dev_logits, (char*)dev_workspace);
  if (rc != PLT_OK) return rc;
  HIP_TRY(hipGetLastError());
  kv->pos = n; kv->started = true;
  return PLT_OK;
}

// ------------------------------------------------------------------------------ hooks
extern "C" int plt_kv_set_position(plt_kv* kv, int32_t pos) {
  if (!kv || pos < 0 || pos > kv->max_ctx) return fail(PLT_EINVAL, "plt_kv_set_position: bad argument");
  launch_pos_set(kv->m->stream, kv->pos_dev, kv->B, pos, 0);
  HIP_TRY(hipGetLastError());
  kv->pos = pos; kv->started = true;
  return PLT_OK;
}

extern "C" size_t plt_kv_export_bytes(const plt_kv* kv, int32_t n) {
  if (!kv || n < 0 || n > kv->max_ctx) { fail(PLT_EINVAL, "plt_kv_export_bytes: bad argument"); return 0; }
  const plt_config& c = kv->m->cfg;
  const size_t w = c.window > 0 ? c.window : 1;
  return ((size_t)2 * c.n_kv_heads * n * c.head_dim + (size_t)2 * kv->n_rings * c.n_kv_heads * w * c.head_dim) * kv->m->kes;
}

template <typename T>
static int kv_xfer(plt_kv* kv, int seq, int layer, int cache, int n, char* host, bool to_host) {
  plt_model* m = kv->m;
  const plt_config& c = m->cfg;
  hipStream_t s = m->stream;
  const int Hkv = c.n_kv_heads, D = c.head_dim, w = c.window > 0 ? c.window : 1, nr = kv->n_rings;
  const size_t total = plt_kv_export_bytes(kv, n);
  T* tmp = nullptr;
  HIP_TRY(hipMalloc((void**)&tmp, total ? total : 256));
  KvView v = kv_view(kv, layer, cache);
  T* ks = (T*)v.k_share + (size_t)seq * Hkv * kv->n_pad * D;
  T* vs = (T*)v.v_share + (size_t)seq * Hkv * kv->n_pad * D;
  T* t_ks = tmp; T* t_vs = tmp + (size_t)Hkv * n * D;
  T* t_kr = t_vs + (size_t)Hkv * n * D; T* t_vr = t_kr + (size_t)nr * Hkv * w * D;
  T* kr = nr ? (T*)v.k_ring + (size_t)seq * nr * Hkv * kv->w_pad * D : nullptr;
  T* vr = nr ? (T*)v.v_ring + (size_t)seq * nr * Hkv * kv->w_pad * D : nullptr;
  hipError_t e = hipSuccess;
  if (to_host) {
    if (n > 0) launch_unpack_k<T>(s, ks, t_ks, Hkv, n, kv->n_pad, D);
    if (n > 0) launch_unpack_v<T>(s, vs, t_vs, Hkv, n, kv->n_pad, D);
    if (nr) launch_unpack_k<T>(s, kr, t_kr, nr * Hkv, w, kv->w_pad, D);
    if (nr) launch_unpack_v<T>(s, vr, t_vr, nr * Hkv, w, kv->w_pad, D);
    if (e == hipSuccess) e = hipMemcpyAsync(host, tmp, total, hipMemcpyDeviceToHost, s);
  } else {
    e = hipMemcpyAsync(tmp, host, total, hipMemcpyHostToDevice, s);
    if (e == hipSuccess && n > 0) {
      // pack into the first whole tiles of each stream (stream stride n_pad positions)
      for (int h = 0; h < Hkv; ++h) {
        launch_pack_k<T>(s, t_ks + (size_t)h * n * D, ks + (size_t)h * kv->n_pad * D, 1, n, pad_kv(n, m->kv8), D);
        launch_pack_v<T>(s, t_vs + (size_t)h * n * D, vs + (size_t)h * kv->n_pad * D, 1, n, pad32(n), D);
      }
    }
    if (nr && e == hipSuccess) {
      launch_pack_k<T>(s, t_kr, kr, nr * Hkv, w, kv->w_pad, D);
      launch_pack_v<T>(s, t_vr, vr, nr * Hkv, w, kv->w_pad, D);
    }
  }
  hipError_t e2 = hipStreamSynchronize(s);
  (void)hipFree(tmp);
  if (e != hipSuccess) return fail(PLT_EHIP, "kv transfer: %s", hipGetErrorString(e));
  if (e2 != hipSuccess) return fail(PLT_EHIP, "kv transfer: %s", hipGetErrorString(e2));
  return PLT_OK;
}

static int kv_xfer_check(plt_kv* kv, int seq, int layer, int cache, int n, const void* host, size_t nbytes) {
  if (!kv || !host) return fail(PLT_EINVAL, "kv export/import: null argument");
  if (seq < 0 || seq >= kv->B || layer < 0 || layer >= kv->m->cfg.n_layers || cache < 0 || cache >= kv->n_caches ||
      n < 0 || n > kv->max_ctx) return fail(PLT_EINVAL, "kv export/import: index out of range");
  if (nbytes != plt_kv_export_bytes(kv, n)) return fail(PLT_EINVAL, "kv export/import: host buffer must have %zu bytes", plt_kv_export_bytes(kv, n));
  return PLT_OK;
}

extern "C" int plt_kv_export(plt_kv* kv, int32_t seq, int32_t layer, int32_t cache, int32_t n, void* host_dst,
                             size_t host_nbytes) {
  int rc = kv_xfer_check(kv, seq, layer, cache, n, host_dst, host_nbytes);
  if (rc) return rc;
  return kv->m->kes == 1 ? kv_xfer<fp8_t>(kv, seq, layer, cache, n, (char*)host_dst, true)
       : kv->m->kes == 2 ? kv_xfer<bf16_t>(kv, seq, layer, cache, n, (char*)host_dst, true)
                         : kv_xfer<float>(kv, seq, layer, cache, n, (char*)host_dst, true);
}
extern "C" int plt_kv_import(plt_kv* kv, int32_t seq, int32_t layer, int32_t cache, int32_t n,
                             const void* host_src, size_t host_nbytes) {
  int rc = kv_xfer_check(kv, seq, layer, cache, n, host_src, host_nbytes);
  if (rc) return rc;
  return kv->m->kes == 1 ? kv_xfer<fp8_t>(kv, seq, layer, cache, n, (char*)host_src, false)
       : kv->m->kes == 2 ? kv_xfer<bf16_t>(kv, seq, layer, cache, n, (char*)host_src, false)
                         : kv_xfer<float>(kv, seq, layer, cache, n, (char*)host_src, false);
}

static int copy_sync(plt_kv* kv, void* dst, const void* src, size_t bytes, hipMemcpyKind kind) {
  HIP_TRY(hipMemcpyAsync(dst, src, bytes, kind, kv->m->stream));
  HIP_TRY(hipStreamSynchronize(kv->m->stream));
  return PLT_OK;
}
extern "C" int plt_get_carry(plt_kv* kv, float* host_dst, size_t host_nbytes) {
  if (!kv || !host_dst) return fail(PLT_EINVAL, "plt_get_carry: null argument");
  const size_t need = (size_t)kv->B * (kv->m->cfg.n_loops - 1) * kv->m->cfg.d_model * 4;
  if (!is_clp(kv->m->cfg) || host_nbytes != need) return fail(PLT_EINVAL, "plt_get_carry: needs CLP mode and %zu bytes", need);
  return need ? copy_sync(kv, host_dst, kv->carry, need, hipMemcpyDeviceToHost) : PLT_OK;
}
extern "C" int plt_set_carry(plt_kv* kv, const float* host_src, size_t host_nbytes) {
  if (!kv || !host_src) return fail(PLT_EINVAL, "plt_set_carry: null argument");
  const size_t need = (size_t)kv->B * (kv->m->cfg.n_loops - 1) * kv->m->cfg.d_model * 4;
  if (!is_clp(kv->m->cfg) || host_nbytes != need) return fail(PLT_EINVAL, "plt_set_carry: needs CLP mode and %zu bytes", need);
  return need ? copy_sync(kv, kv->carry, host_src, need, hipMemcpyHostToDevice) : PLT_OK;
}
extern "C" int plt_get_hidden(plt_kv* kv, float* host_dst, size_t host_nbytes) {
  if (!kv || !host_dst) return fail(PLT_EINVAL, "plt_get_hidden: null argument");
  const int rows = is_clp(kv->m->cfg) ? kv->B * kv->m->cfg.n_loops : kv->B;
  const size_t need = (size_t)rows * kv->m->cfg.d_model * 4;
  if (host_nbytes != need) return fail(PLT_EINVAL, "plt_get_hidden: host buffer must have %zu bytes", need);
  return copy_sync(kv, host_dst, kv->x, need, hipMemcpyDeviceToHost);
}

// One layer of block f on the decode micro-batch, from a given residual stream (test hook): what the decode step
// does for layer `layer` at the position the next plt_decode_step would consume, cache append included.
template <typename T>
static void debug_layer_t(plt_model* m, plt_kv* kv, int layer) {
  const plt_config& c = m->cfg;
  const int B = kv->B, L = c.n_loops, R = B * L;
  Work wk{kv->x, kv->a, kv->gout, kv->q, kv->z, kv->y, kv->act, nullptr, kv->moe_idx, kv->a_codes, kv->a_scales, kv->act_sc};
  KvView none{}; none.b0 = 0;
  RowMap rm{0, L, 0, kv->pos_dev};
  norm_to_a<T>(m, wk, nullptr, 0, 0, m->layers[layer].norm1, R);
  const int variant = c.mode == PLT_MODE_CLP ? V_PLT : (c.mode == PLT_MODE_CLP_SHARE_ONLY ? V_SHARE_ONLY : V_OWN_KV);
  stack_pass<T>(m, kv, wk, R, rm, 0, variant, none, 0, 0, L, nullptr, layer, layer + 1);
}
extern "C" int plt_debug_layer(plt_model* m, plt_kv* kv, int32_t layer, const float* host_x_in, float* host_x_out,
                               size_t host_nbytes) {
  if (!m || !kv || kv->m != m || !host_x_in || !host_x_out) return fail(PLT_EINVAL, "plt_debug_layer: bad argument");
  const plt_config& c = m->cfg;
  if (!is_clp(c)) return fail(PLT_EINVAL, "plt_debug_layer: not available in vanilla-loop mode");
  if (layer < 0 || layer >= c.n_layers) return fail(PLT_EINVAL, "plt_debug_layer: layer out of range");
  if (!kv->started) return fail(PLT_ESTATE, "plt_debug_layer: plt_prefill (or plt_kv_set_position) must come first");
  if (kv->pos >= kv->max_ctx) return fail(PLT_ECTXFULL, "plt_debug_layer: context full (%d positions)", kv->max_ctx);
  const size_t need = (size_t)kv->B * c.n_loops * c.d_model * 4;
  if (host_nbytes != need) return fail(PLT_EINVAL, "plt_debug_layer: host buffers must have %zu bytes", need);
  int rc = copy_sync(kv, kv->x, host_x_in, need, hipMemcpyHostToDevice);
  if (rc != PLT_OK) return rc;
  if (m->mx && c.n_experts == 0 && !kv->dbg_codes) {        // capture slots of the four quantised projection inputs
    const int maxK = mx_max_k(c), R = kv->B * c.n_loops;
    kv->dbg_codes_slot = align256((size_t)R * maxK); kv->dbg_scales_slot = align256((size_t)R * mx_ascale_row_bytes(maxK));
    HIP_TRY(hipMalloc((void**)&kv->dbg_codes, 4 * kv->dbg_codes_slot));
    HIP_TRY(hipMalloc((void**)&kv->dbg_scales, 4 * kv->dbg_scales_slot));
  }
  kv->dbg_on = kv->dbg_codes != nullptr;
  if (c.dtype == PLT_BF16) debug_layer_t<bf16_t>(m, kv, layer); else debug_layer_t<float>(m, kv, layer);
  kv->dbg_on = false;
  HIP_TRY(hipGetLastError());
  return copy_sync(kv, host_x_out, kv->x, need, hipMemcpyDeviceToHost);
}

extern "C" int plt_debug_act_codes(plt_kv* kv, int32_t which, uint8_t* host_codes, size_t codes_nbytes,
                                   uint8_t* host_scales, size_t scales_nbytes) {
  if (!kv || !host_codes || !host_scales || which < 0 || which > 3) return fail(PLT_EINVAL, "plt_debug_act_codes: bad argument");
  const plt_config& c = kv->m->cfg;
  if (!kv->dbg_codes) return fail(PLT_ESTATE, "plt_debug_act_codes: needs a dense low-bit model and a plt_debug_layer call first");
  const int K = which == 1 ? c.n_heads * c.head_dim : (which == 3 ? c.ffn_hidden : c.d_model), R = kv->B * c.n_loops;
  const size_t nc = (size_t)R * K, ns = (size_t)R * mx_ascale_row_bytes(K);
  if (codes_nbytes != nc || scales_nbytes != ns) return fail(PLT_EINVAL, "plt_debug_act_codes: buffers must have %zu and %zu bytes", nc, ns);
  int rc = copy_sync(kv, host_codes, kv->dbg_codes + which * kv->dbg_codes_slot, nc, hipMemcpyDeviceToHost);
  if (rc != PLT_OK) return rc;
  return copy_sync(kv, host_scales, kv->dbg_scales + which * kv->dbg_scales_slot, ns, hipMemcpyDeviceToHost);
}

// ---- kernel-only hooks ----
__global__ void k_sum_slabs(const float* __restrict__ p, float* __restrict__ c, int S, size_t n);
extern "C" int32_t plt_attn_pad32(int32_t n) { return pad32(n); }
extern "C" int32_t plt_attn_pad(int32_t dtype, int32_t n) { return pad_kv(n, dtype == PLT_FP8_E4M3); }

extern "C" size_t plt_attn_scratch_bytes(int32_t B, int32_t L, int32_t Hq, int32_t Hkv, int32_t D) {
  if (B < 1 || L < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || (D != 64 && D != 128)) { fail(PLT_EINVAL, "plt_attn_scratch_bytes: bad shape"); return 0; }
  size_t s = attn_mfma_scratch_bytes(B, L, Hq, Hkv, D);
  size_t p = align256((size_t)B * 4);
  return s > p ? s : p;
}

// shared by plt_attn_decode and plt_attn_decode_static: argument checks, then the launches on `scratch`
static int attn_decode_checked(const char* who, int32_t dtype, int32_t B, int32_t L, int32_t Hq, int32_t Hkv, int32_t D,
                               int32_t n_alloc, int32_t n_ctx, int32_t w, int32_t n_ring, const void* q,
                               const void* k_share, const void* v_share, const void* k_ring, const void* v_ring,
                               const float* z, void* y, void* scratch, size_t scratch_bytes, bool exact_scratch,
                               int32_t n_splits, void* hip_stream) {
  if (dtype != PLT_F32 && dtype != PLT_BF16 && dtype != PLT_FP8_E4M3) return fail(PLT_EINVAL, "%s: unknown dtype", who);
  const bool kv8 = dtype == PLT_FP8_E4M3;
  if (B < 1 || L < 1 || L > 16 || Hq < 1 || Hkv < 1 || Hq % Hkv || (D != 64 && D != 128))
    return fail(PLT_EINVAL, "%s: bad shape", who);
  if (n_ctx < 1 || n_ctx > n_alloc) return fail(PLT_EINVAL, "%s: need 1 <= n_ctx <= n_alloc", who);
  if (L > 1 && (w < 1 || n_ring < 1 || n_ring > w)) return fail(PLT_EINVAL, "%s: need 1 <= n_ring <= w", who);
  if (!q || !k_share || !v_share || !y || !scratch || (L > 1 && (!k_ring || !v_ring || !z)))
    return fail(PLT_EINVAL, "%s: null pointer", who);
  if ((long)B * L > 60000) return fail(PLT_EINVAL, "%s: B * L too large", who);
  hipStream_t s = (hipStream_t)hip_stream;
  KvView v{};
  v.k_share = (void*)k_share; v.v_share = (void*)v_share; v.k_ring = (void*)k_ring; v.v_ring = (void*)v_ring;
  v.n_pad = pad_kv(n_alloc, kv8); v.w_pad = pad_kv(w > 0 ? w : 1, kv8); v.w = w > 0 ? w : 1; v.n_rings = L - 1; v.b0 = 0;
  Dims dm{B, L, Hq, Hkv, D, 0, 0, 0};
  if (dtype == PLT_BF16 || kv8) {
    if (n_splits <= 0) n_splits = attn_mfma_default_splits(B, Hkv, L, Hq / Hkv, n_ctx, kv8);
    if (n_splits > 64) n_splits = 64;
    // exact_scratch: the buffer is laid out for exactly the splits of this call (the library's own static buffer);
    // otherwise for the 64 splits plt_attn_scratch_bytes sizes a caller's buffer for
    const int layout_splits = exact_scratch ? n_splits : 64;
    const size_t need = attn_mfma_scratch_bytes(B, L, Hq, Hkv, D, layout_splits);
    if (scratch_bytes < need) return fail(PLT_ENOMEM, "%s: needs %zu bytes of scratch for %d splits, %zu available", who, need, n_splits, scratch_bytes);
    launch_attn_decode_mfma(s, (const bf16_t*)q, z, (bf16_t*)y, v, nullptr, n_ctx, L > 1 ? n_ring : 0, dm, 0,
                            scratch, n_splits, 0, 0, kv8, layout_splits);
  } else {
    if (scratch_bytes < align256((size_t)B * 4)) return fail(PLT_ENOMEM, "%s: scratch too small", who);
    if (L > 1 && n_ring != (n_ctx < w ? n_ctx : w))
      return fail(PLT_EINVAL, "%s: float path needs n_ring == min(n_ctx, w)", who);
    launch_pos_set(s, (int32_t*)scratch, B, n_ctx - 1, 0);
    RowMap rm{0, L, 0, (const int32_t*)scratch};
    launch_attn_f32(s, (const float*)q, z, (float*)y, v, rm, B * L, dm, 0);
  }
  HIP_TRY(hipGetLastError());
  return PLT_OK;
}

extern "C" int plt_attn_decode(int32_t dtype, int32_t B, int32_t L, int32_t Hq, int32_t Hkv, int32_t D,
                               int32_t n_alloc, int32_t n_ctx, int32_t w, int32_t n_ring, const void* q,
                               const void* k_share, const void* v_share, const void* k_ring, const void* v_ring,
                               const float* z, void* y, void* scratch, size_t scratch_bytes, int32_t n_splits,
                               void* hip_stream) {
  return attn_decode_checked("plt_attn_decode", dtype, B, L, Hq, Hkv, D, n_alloc, n_ctx, w, n_ring, q, k_share, v_share,
                             k_ring, v_ring, z, y, scratch, scratch_bytes, false, n_splits, hip_stream);
}

extern "C" int plt_attn_decode_static(int32_t dtype, int32_t B, int32_t L, int32_t Hq, int32_t Hkv, int32_t D,
                                      int32_t n_alloc, int32_t n_ctx, int32_t w, int32_t n_ring, const void* q,
                                      const void* k_share, const void* v_share, const void* k_ring, const void* v_ring,
                                      const float* z, void* y, int32_t n_splits, void* hip_stream) {
  void* sp = nullptr;
  const int rc = static_scratch(&sp);        // a table look-up after the first call on this device
  if (rc != PLT_OK) return rc;
  // same checks and launches as plt_attn_decode; the records are laid out for exactly this call's splits, every
  // record a launch reads is written by the same launch first (nothing has to start at zero), and a shape whose
  // records exceed the array is refused
  return attn_decode_checked("plt_attn_decode_static", dtype, B, L, Hq, Hkv, D, n_alloc, n_ctx, w, n_ring, q, k_share,
                             v_share, k_ring, v_ring, z, y, sp, (size_t)PLT_ATTN_STATIC_SCRATCH_BYTES, true, n_splits,
                             hip_stream);
}

extern "C" int64_t plt_attn_k_index(int32_t dtype, int32_t pos, int32_t f, int32_t D) {
  if (pos < 0 || f < 0 || f >= D || (D != 64 && D != 128)) return -1;
  if (dtype == PLT_F32) return (int64_t)kblk_index<float>(pos, f, D);
  if (dtype == PLT_BF16) return (int64_t)kblk_index<bf16_t>(pos, f, D);
  if (dtype == PLT_FP8_E4M3) return (int64_t)kblk_index<fp8_t>(pos, f, D);
  return -1;
}

extern "C" int64_t plt_attn_v_index(int32_t dtype, int32_t pos, int32_t d, int32_t D) {
  if (pos < 0 || d < 0 || d >= D || (D != 64 && D != 128)) return -1;
  if (dtype == PLT_F32) return (int64_t)vblk_index<float>(pos, d, D);
  if (dtype == PLT_BF16) return (int64_t)vblk_index<bf16_t>(pos, d, D);
  if (dtype == PLT_FP8_E4M3) return (int64_t)vblk_index<fp8_t>(pos, d, D);
  return -1;
}

extern "C" int plt_attn_pack_k(int32_t dtype, int32_t S, int32_t n, int32_t D, const void* src, void* dst,
                               void* hip_stream) {
  if ((dtype != PLT_F32 && dtype != PLT_BF16 && dtype != PLT_FP8_E4M3) || S < 1 || S > 65535 || n < 1 || D < 1 || !src || !dst)
    return fail(PLT_EINVAL, "plt_attn_pack_k: bad argument");
  if (dtype == PLT_FP8_E4M3) launch_pack_k<fp8_t>((hipStream_t)hip_stream, (const fp8_t*)src, (fp8_t*)dst, S, n, pad_kv(n, true), D);
  else if (dtype == PLT_BF16) launch_pack_k<bf16_t>((hipStream_t)hip_stream, (const bf16_t*)src, (bf16_t*)dst, S, n, pad32(n), D);
  else launch_pack_k<float>((hipStream_t)hip_stream, (const float*)src, (float*)dst, S, n, pad32(n), D);
  HIP_TRY(hipGetLastError());
  return PLT_OK;
}
extern "C" int plt_attn_pack_v(int32_t dtype, int32_t S, int32_t n, int32_t D, const void* src, void* dst,
                               void* hip_stream) {
  if ((dtype != PLT_F32 && dtype != PLT_BF16 && dtype != PLT_FP8_E4M3) || S < 1 || S > 65535 || n < 1 || D < 1 || !src || !dst)
    return fail(PLT_EINVAL, "plt_attn_pack_v: bad argument");
  if (dtype == PLT_FP8_E4M3) launch_pack_v<fp8_t>((hipStream_t)hip_stream, (const fp8_t*)src, (fp8_t*)dst, S, n, pad_kv(n, true), D);
  else if (dtype == PLT_BF16) launch_pack_v<bf16_t>((hipStream_t)hip_stream, (const bf16_t*)src, (bf16_t*)dst, S, n, pad32(n), D);
  else launch_pack_v<float>((hipStream_t)hip_stream, (const float*)src, (float*)dst, S, n, pad32(n), D);
  HIP_TRY(hipGetLastError());
  return PLT_OK;
}

extern "C" int64_t plt_moe_weight_index(int32_t n, int32_t k, int32_t K) {
  if (n < 0 || k < 0 || K < 32 || (K & 31) || k >= K) return -1;
  return (int64_t)moe_wtile_index(n, k, K);
}

extern "C" size_t plt_moe_scratch_bytes(int32_t dtype, int32_t R, int32_t d, int32_t F, int32_t E, int32_t k) {
  if ((dtype != PLT_F32 && dtype != PLT_BF16) || R < 1 || d < 1 || F < 1 || E < 1 || E > 256 || k < 1 || k > E || k > 32) {
    fail(PLT_EINVAL, "plt_moe_scratch_bytes: bad argument"); return 0;
  }
  const size_t es = dtype == PLT_BF16 ? 2 : 4;
  return moe_index_bytes(R, k, E) + align256((size_t)R * k * F * es) + align256((size_t)k * R * d * 4);
}

extern "C" int plt_moe_ffn(int32_t dtype, int32_t R, int32_t d, int32_t F, int32_t E, int32_t k, const void* a,
                           const void* router, const void* wgu, const void* wdown, float* y, int32_t* sel_e,
                           float* sel_p, void* scratch, size_t scratch_bytes, void* hip_stream) {
  const size_t need = plt_moe_scratch_bytes(dtype, R, d, F, E, k);
  if (need == 0) return fail(PLT_EINVAL, "plt_moe_ffn: bad shape or dtype");
  if (dtype == PLT_BF16 && (d % 64 || F % 64)) return fail(PLT_EINVAL, "plt_moe_ffn: bf16 needs d and F to be multiples of 64");
  if ((long)R * k > 2000000L) return fail(PLT_EINVAL, "plt_moe_ffn: R * k too large");
  if (!a || !router || !wgu || !wdown || !y || !sel_e || !sel_p || !scratch) return fail(PLT_EINVAL, "plt_moe_ffn: null pointer");
  if (scratch_bytes < need || (((uintptr_t)scratch) & 255)) return fail(PLT_ENOMEM, "plt_moe_ffn: scratch too small or not 256-byte aligned");
  hipStream_t s = (hipStream_t)hip_stream;
  const size_t es = dtype == PLT_BF16 ? 2 : 4;
  char* base = (char*)scratch;
  MoeIndex mi = moe_index_carve(base, R, k, E);
  void* act = base + moe_index_bytes(R, k, E);
  float* slabs = (float*)((char*)act + align256((size_t)R * k * F * es));
  if (dtype == PLT_BF16)
    launch_moe_ffn<bf16_t>(s, (const bf16_t*)a, (const bf16_t*)router, (const bf16_t*)wgu, (const bf16_t*)wdown, (bf16_t*)act,
                           slabs, mi, R, d, F, E, k);
  else
    launch_moe_ffn<float>(s, (const float*)a, (const float*)router, (const float*)wgu, (const float*)wdown, (float*)act,
                          slabs, mi, R, d, F, E, k);
  const size_t n = (size_t)R * d;
  hipLaunchKernelGGL(k_sum_slabs, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const float*)slabs, y, k, n);
  HIP_TRY(hipMemcpyAsync(sel_e, mi.sel_e, (size_t)R * k * 4, hipMemcpyDeviceToDevice, s));
  HIP_TRY(hipMemcpyAsync(sel_p, mi.sel_p, (size_t)R * k * 4, hipMemcpyDeviceToDevice, s));
  HIP_TRY(hipGetLastError());
  return PLT_OK;
}

// ---- low-bit (microscaling) projection hooks ----
static bool mx_shape_ok(int N, int K) { return N >= 16 && (N % 16) == 0 && K >= 128 && (K % 128) == 0; }
extern "C" size_t plt_mx_weight_code_bytes(int32_t N, int32_t K) {
  if (!mx_shape_ok(N, K)) { fail(PLT_EINVAL, "plt_mx_weight_code_bytes: N must be a multiple of 16, K of 128"); return 0; }
  return (size_t)N * K / 2;
}
extern "C" size_t plt_mx_weight_scale_bytes(int32_t N, int32_t K) {
  if (!mx_shape_ok(N, K)) { fail(PLT_EINVAL, "plt_mx_weight_scale_bytes: N must be a multiple of 16, K of 128"); return 0; }
  return mx_wscale_bytes(N, K);
}
extern "C" size_t plt_mx_act_scale_bytes(int32_t M, int32_t K) {
  if (M < 1 || K < 32 || (K % 32)) { fail(PLT_EINVAL, "plt_mx_act_scale_bytes: bad shape"); return 0; }
  return (size_t)M * mx_ascale_row_bytes(K);
}
extern "C" int64_t plt_mx_weight_code_index(int32_t n, int32_t k, int32_t K) {
  if (n < 0 || k < 0 || k >= K || K % 128) return -1;
  return (int64_t)mx_wcode_index(n, k, K);
}
extern "C" int64_t plt_mx_weight_scale_index(int32_t n, int32_t b, int32_t K) {
  if (n < 0 || b < 0 || b * 32 >= K || K % 128) return -1;
  return (int64_t)mx_wscale_index(n, b, K);
}
extern "C" int32_t plt_mx_act_scale_index(int32_t b) { return b < 0 ? -1 : mx_ascale_index(b); }

extern "C" int plt_mx_quantize_weights(int32_t N, int32_t K, const void* src_bf16, void* codes, void* scales, void* hip_stream) {
  if (!mx_shape_ok(N, K) || !src_bf16 || !codes || !scales) return fail(PLT_EINVAL, "plt_mx_quantize_weights: bad argument (N %% 16, K %% 128)");
  if ((((uintptr_t)codes) | ((uintptr_t)scales) | ((uintptr_t)src_bf16)) & 15) return fail(PLT_EINVAL, "plt_mx_quantize_weights: pointers must be 16-byte aligned");
  hipStream_t s = (hipStream_t)hip_stream;
  HIP_TRY(hipMemsetAsync(scales, 0, mx_wscale_bytes(N, K), s));      // scale bytes of chunks beyond K stay 0
  launch_mx_quant_w(s, (const bf16_t*)src_bf16, (uint8_t*)codes, (uint8_t*)scales, N, K);
  HIP_TRY(hipGetLastError());
  return PLT_OK;
}
extern "C" int plt_mx_quantize_act(int32_t dtype, int32_t M, int32_t K, const void* src, void* codes, void* scales, void* hip_stream) {
  if ((dtype != PLT_F32 && dtype != PLT_BF16) || M < 1 || K < 32 || (K % 32) || !src || !codes || !scales)
    return fail(PLT_EINVAL, "plt_mx_quantize_act: bad argument (K %% 32)");
  if ((((uintptr_t)codes) | ((uintptr_t)src)) & 15) return fail(PLT_EINVAL, "plt_mx_quantize_act: pointers must be 16-byte aligned");
  hipStream_t s = (hipStream_t)hip_stream;
  if (dtype == PLT_F32) launch_mx_quant_a<float>(s, (const float*)src, (uint8_t*)codes, (uint8_t*)scales, M, K);
  else launch_mx_quant_a<bf16_t>(s, (const bf16_t*)src, (uint8_t*)codes, (uint8_t*)scales, M, K);
  HIP_TRY(hipGetLastError());
  return PLT_OK;
}
extern "C" size_t plt_gemm_mx_scratch_bytes(int32_t M, int32_t N, int32_t K) {
  if (M < 1 || !mx_shape_ok(N, K)) { fail(PLT_EINVAL, "plt_gemm_mx_scratch_bytes: bad shape"); return 0; }
  return align256((size_t)gemm_mx_splits(M, N, K) * M * N * 4);
}
extern "C" int plt_gemm_mx(int32_t M, int32_t N, int32_t K, const void* a_codes, const void* a_scales, const void* w_codes,
                           const void* w_scales, float* c, void* scratch, size_t scratch_bytes, void* hip_stream) {
  if (M < 1 || M > 128 * 65535 || !mx_shape_ok(N, K) || !a_codes || !a_scales || !w_codes || !w_scales || !c)
    return fail(PLT_EINVAL, "plt_gemm_mx: bad argument (N %% 16, K %% 128)");
  if ((((uintptr_t)a_codes) | ((uintptr_t)a_scales) | ((uintptr_t)w_codes) | ((uintptr_t)w_scales) | ((uintptr_t)c)) & 15)
    return fail(PLT_EINVAL, "plt_gemm_mx: pointers must be 16-byte aligned");
  hipStream_t s = (hipStream_t)hip_stream;
  const int S = gemm_mx_splits(M, N, K);
  if (S == 1) {
    launch_gemm_mx(s, (const uint8_t*)a_codes, (const uint8_t*)a_scales, (const uint8_t*)w_codes, (const uint8_t*)w_scales, c, M, N, K);
  } else {
    if (!scratch || scratch_bytes < plt_gemm_mx_scratch_bytes(M, N, K)) return fail(PLT_ENOMEM, "plt_gemm_mx: scratch too small");
    launch_gemm_mx(s, (const uint8_t*)a_codes, (const uint8_t*)a_scales, (const uint8_t*)w_codes, (const uint8_t*)w_scales,
                   (float*)scratch, M, N, K);
    const size_t n = (size_t)M * N;
    hipLaunchKernelGGL(k_sum_slabs, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const float*)scratch, c, S, n);
  }
  HIP_TRY(hipGetLastError());
  return PLT_OK;
}

extern "C" size_t plt_gemm_mx_swiglu_scratch_bytes(int32_t M, int32_t F, int32_t K) {
  if (M < 1 || F < 32 || (F % 32) || !mx_shape_ok(2 * F, K)) { fail(PLT_EINVAL, "plt_gemm_mx_swiglu_scratch_bytes: bad shape"); return 0; }
  return gemm_mx_swiglu_rows_applies(M, F, K) ? 256 : align256((size_t)gemm_mx_splits(M, 2 * F, K) * M * 2 * F * 4);
}
extern "C" int plt_gemm_mx_swiglu(int32_t M, int32_t F, int32_t K, const void* a_codes, const void* a_scales, const void* w_codes,
                                  const void* w_scales, void* h_codes, void* h_scales, void* scratch, size_t scratch_bytes,
                                  void* hip_stream) {
  if (M < 1 || M > 128 * 65535 || F < 32 || (F % 32) || !mx_shape_ok(2 * F, K) || !a_codes || !a_scales || !w_codes || !w_scales ||
      !h_codes || !h_scales)
    return fail(PLT_EINVAL, "plt_gemm_mx_swiglu: bad argument (F %% 32, K %% 128)");
  if ((((uintptr_t)a_codes) | ((uintptr_t)a_scales) | ((uintptr_t)w_codes) | ((uintptr_t)w_scales) | ((uintptr_t)h_codes) |
       ((uintptr_t)h_scales)) & 15)
    return fail(PLT_EINVAL, "plt_gemm_mx_swiglu: pointers must be 16-byte aligned");
  if (h_codes == a_codes || h_scales == a_scales) return fail(PLT_EINVAL, "plt_gemm_mx_swiglu: the result must not overwrite the operand");
  hipStream_t s = (hipStream_t)hip_stream;
  if (gemm_mx_swiglu_rows_applies(M, F, K)) {
    launch_gemm_mx_swiglu_rows(s, (const uint8_t*)a_codes, (const uint8_t*)a_scales, (const uint8_t*)w_codes, (const uint8_t*)w_scales,
                               (uint8_t*)h_codes, (uint8_t*)h_scales, M, F, K);
  } else {
    if (!scratch || scratch_bytes < plt_gemm_mx_swiglu_scratch_bytes(M, F, K)) return fail(PLT_ENOMEM, "plt_gemm_mx_swiglu: scratch too small");
    launch_gemm_mx(s, (const uint8_t*)a_codes, (const uint8_t*)a_scales, (const uint8_t*)w_codes, (const uint8_t*)w_scales,
                   (float*)scratch, M, 2 * F, K);
    launch_silu_mul_mx(s, (const float*)scratch, gemm_mx_splits(M, 2 * F, K), (size_t)M * 2 * F, (uint8_t*)h_codes, (uint8_t*)h_scales, M, F);
  }
  HIP_TRY(hipGetLastError());
  return PLT_OK;
}

// plain copy, 16 bytes per lane per iteration: the reference point for HBM counters and the
// practical bandwidth ceiling the attention kernel is compared with
__global__ __launch_bounds__(256) void k_stream_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) dst[i] = src[i];
}

// read-only counterpart: every workgroup walks one contiguous chunk (like one K/V stream), eight
// 16-byte non-temporal loads in flight per lane (the fastest plain read found on this part: 512
// workgroups, 64 KB in flight per compute unit); every lane folds what it reads and stores one word
__global__ __launch_bounds__(256) void k_stream_read(const uint4* __restrict__ src, unsigned* __restrict__ out, size_t n16) {
  const size_t per = n16 / gridDim.x;
  const uint4* p = src + (size_t)blockIdx.x * per;
  unsigned acc = 0;
  size_t i = threadIdx.x;
  for (; i + 7 * 256 < per; i += 8 * 256) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = ldg16_stream(p + i + u * 256);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < per; i += 256) { uint4 a = p[i]; acc ^= a.x ^ a.y ^ a.z ^ a.w; }
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

extern "C" int plt_stream_read(const void* dev_src, size_t nbytes, void* dev_out, size_t out_bytes, void* hip_stream) {
  const size_t blocks = 256 * 2, gran = 32768, out_need = (size_t)2 << 20;
  if (!dev_src || !dev_out || nbytes == 0 || (nbytes % gran) || (((uintptr_t)dev_src) & 15) || out_bytes < out_need)
    return fail(PLT_EINVAL, "plt_stream_read: need a multiple of %zu bytes, 16-byte alignment and an output buffer of %zu bytes",
                gran, out_need);
  hipLaunchKernelGGL(k_stream_read, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream,
                     (const uint4*)dev_src, (unsigned*)dev_out, nbytes / 16);
  HIP_TRY(hipGetLastError());
  return PLT_OK;
}

extern "C" int plt_stream_copy(void* dev_dst, const void* dev_src, size_t nbytes, void* hip_stream) {
  if (!dev_dst || !dev_src || nbytes == 0 || (nbytes & 15) || (((uintptr_t)dev_dst | (uintptr_t)dev_src) & 15))
    return fail(PLT_EINVAL, "plt_stream_copy: pointers and size must be non-null multiples of 16 bytes");
  const size_t n16 = nbytes / 16;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  hipLaunchKernelGGL(k_stream_copy, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream,
                     (const uint4*)dev_src, (uint4*)dev_dst, n16);
  HIP_TRY(hipGetLastError());
  return PLT_OK;
}

__global__ void k_sum_slabs(const float* __restrict__ p, float* __restrict__ c, int S, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float v = 0.f;
  for (int s = 0; s < S; ++s) v += p[(size_t)s * n + i];
  c[i] = v;
}

extern "C" size_t plt_gemm_scratch_bytes(int32_t M, int32_t N, int32_t K) {
  if (M < 1 || N < 1 || K < 1) { fail(PLT_EINVAL, "plt_gemm_scratch_bytes: bad shape"); return 0; }
  return align256((size_t)gemm_bf16_splits_any(M, N, K) * M * N * 4);
}

extern "C" int plt_gemm_residual(int32_t M, int32_t N, int32_t K, const void* a, const void* w, float* x, void* hip_stream) {
  if (M < 1 || N < 1 || K < 1 || !a || !w || !x) return fail(PLT_EINVAL, "plt_gemm_residual: bad argument");
  if ((long)M > 256L * 65535 || !gemm_big_applies(M, N, K))
    return fail(PLT_EINVAL, "plt_gemm_residual: only shapes that take the 256 x 256 tile kernel (M >= 512, >= 200 tiles, K %% 64 == 0)");
  launch_gemm_big_resid((hipStream_t)hip_stream, (const bf16_t*)a, (const bf16_t*)w, x, M, N, K);
  HIP_TRY(hipGetLastError());
  return PLT_OK;
}

extern "C" int plt_gemm(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* a, const void* w, float* c,
                        void* scratch, size_t scratch_bytes, void* hip_stream) {
  if ((dtype != PLT_F32 && dtype != PLT_BF16) || M < 1 || N < 1 || K < 1 || !a || !w || !c)
    return fail(PLT_EINVAL, "plt_gemm: bad argument");
  if ((long)M > 128L * 65535 || (long)N > 64L * 2147483647L) return fail(PLT_EINVAL, "plt_gemm: too large");
  hipStream_t s = (hipStream_t)hip_stream;
  if (dtype == PLT_F32) {
    launch_gemm_f32(s, (const float*)a, (const float*)w, c, M, N, K);
  } else {
    if (K % 64) return fail(PLT_EINVAL, "plt_gemm: bf16 needs K to be a multiple of 64");
    const int S = gemm_bf16_splits_any(M, N, K);
    if (S == 1) {
      launch_gemm_bf16_any(s, (const bf16_t*)a, (const bf16_t*)w, c, M, N, K);
    } else {
      if (!scratch || scratch_bytes < plt_gemm_scratch_bytes(M, N, K)) return fail(PLT_ENOMEM, "plt_gemm: scratch too small");
      launch_gemm_bf16_any(s, (const bf16_t*)a, (const bf16_t*)w, (float*)scratch, M, N, K);
      const size_t n = (size_t)M * N;
      hipLaunchKernelGGL(k_sum_slabs, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (const float*)scratch, c, S, n);
    }
  }
  HIP_TRY(hipGetLastError());
  return PLT_OK;
}
