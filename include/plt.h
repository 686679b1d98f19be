/*
 * plt.h -- C ABI of the MI355X (gfx950) implementation of the Parallel Loop Transformer's
 * cross-loop-parallel (CLP) decode path (arxiv 2510.24824).
 *
 * Conventions
 *   - Every function returns 0 (PLT_OK) or a negative plt_status; plt_last_error() gives a
 *     thread-local message for the last failure.  No C++ exception crosses this boundary.
 *   - "dev" pointers are HIP device pointers owned by the caller (the library never frees
 *     them); "host" pointers are ordinary host memory.  The stream handed to plt_init is the
 *     caller's hipStream_t (NULL = default stream); all work is asynchronous on it except the
 *     export / import / debug hooks (the ones that take host pointers), which synchronise the stream.
 *     plt_init and plt_kv_alloc are the only calls that allocate device memory (small tables and
 *     the per-step activation scratch); plt_prefill and plt_decode_step allocate nothing, never
 *     synchronise and clear memory with kernels only, so their launches may be captured in a HIP graph.
 *   - Matrices are row-major [out_features, in_features] (y = W x).  dtype PLT_F32 keeps
 *     weights, caches and GEMM inputs in float; PLT_BF16 keeps them in bfloat16 with float
 *     accumulation, a float residual stream and float softmax statistics.
 *   - Requirements: head_dim in {64, 128}; n_heads % n_kv_heads == 0; for PLT_BF16 also
 *     d_model % 64 == 0 and ffn_hidden % 64 == 0.  Anything else -> PLT_EINVAL.
 *   - One model may serve several plt_kv objects, but calls that share a model or a kv
 *     object must not overlap in time (they share scratch memory).
 *
 * Model statement (sections of the paper in brackets).  Block f is a pre-norm decoder
 * stack (RMSNorm, attention, residual, RMSNorm, SwiGLU, residual) whose weights are reused
 * by every loop.  Loop 1 is an ordinary causal transformer pass whose rotated keys and
 * values form the single shared cache K_share, V_share [Sec. 2.2.2].  Loop l >= 2 at
 * position p takes e_p + H^(l-1)[p-1] as input [Alg. 2; Sec. 2.2.1] and its attention is
 * global attention over K_share, V_share[0..p] plus sliding-window attention over its own
 * last w keys/values, merged per head by g = sigmoid(<q_h, wg_h> + bg_h):
 * y = g * y_local + (1 - g) * y_global [Alg. 3; Eq. 2].  While decoding, the L loop stages
 * of one position form one micro-batch of L rows and run as a single pass [Alg. 1].
 * With n_experts > 0 the feed-forward of every layer is a mixture of SwiGLU experts [appendix,
 * "MoE Models Recipe": k of E experts per token].  The paper does not print the router; the reading
 * taken is: logits r = W_r b on the normed row b, p = softmax(r) over all E experts, the k experts
 * with the largest p are evaluated (equal p: lowest index first; softmax is monotone, so the device
 * takes the same decision on the float logits r) and their outputs are summed with weights p_e as
 * they are (not renormalised).
 */
#ifndef PLT_H_
#define PLT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PLT_OK = 0,
  PLT_EINVAL = -1,   /* bad argument or unsupported configuration           */
  PLT_ENOMEM = -2,   /* a caller buffer is too small, or hipMalloc failed    */
  PLT_ECTXFULL = -3, /* the next position would exceed max_ctx (no state change) */
  PLT_EHIP = -4,     /* a HIP runtime call failed                            */
  PLT_ESTATE = -5    /* call order violated (e.g. decode before prefill)     */
} plt_status;

enum { PLT_F32 = 0, PLT_BF16 = 1 };
/* Cache-only element type: the 8-bit float e4m3 (1 sign, 4 exponent bits with bias 7, 3 mantissa
 * bits, no infinities, largest value 448; the OCP "e4m3fn" encoding).  The paper serves its
 * models with FP8 self-attention [inference efficiency evaluation recipe]; here that is a
 * storage format: every K (after RoPE) and V is rounded once, to nearest even with saturation
 * at +-448 and unit scale, when it enters a cache; attention reads the stored values exactly
 * and keeps bf16 queries / softmax weights and float statistics.  bf16 models only. */
enum { PLT_FP8_E4M3 = 2 };
/* Weight-only element type of the low-bit projections (e2m1 in blocks of 32 with power-of-two scales). */
enum { PLT_MXFP4 = 3 };

/* mode: which schedule / cache organisation the model object runs.                        */
enum {
  PLT_MODE_CLP = 0,          /* PLT: Alg. 1 decoding, shared first-loop KV, gated window    */
  PLT_MODE_VANILLA_LOOP = 2, /* Eq. (1): L serial passes per token, one full cache per loop,
                                no shift, no gate, no window (the paper's baseline row 2)   */
  PLT_MODE_CLP_SHARE_ONLY = 3, /* Table 1 row 4: cross-loop parallel, non-first loops attend the
                                shared first-loop cache only (no own K/V, no window, no gate) */
  PLT_MODE_CLP_OWN_KV = 4    /* Table 1 row 3: cross-loop parallel, every loop keeps and attends
                                its own full cache (no sharing, no window, no gate)         */
};

typedef struct plt_config {
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, ffn_hidden, vocab;
  int32_t n_loops;        /* L >= 1; L == 1 is the non-looped transformer                   */
  int32_t window;         /* w >= 1 (ignored when L == 1 or in vanilla-loop mode)           */
  int32_t dtype;          /* PLT_F32 or PLT_BF16                                            */
  int32_t mode;           /* PLT_MODE_*                                                     */
  int32_t tie_embeddings; /* 1: classifier head = embedding matrix                          */
  float rope_theta;       /* rotary base (10000)                                            */
  float norm_eps;         /* RMSNorm epsilon                                                */
  int32_t kv_dtype;       /* 0: caches hold the model dtype; PLT_FP8_E4M3: caches hold e4m3
                             (needs dtype == PLT_BF16; halves the KV bytes of Table 1)      */
  int32_t n_experts;      /* E: 0 = dense SwiGLU feed-forward; 1..256 = mixture of E SwiGLU
                             experts of hidden size ffn_hidden each [appendix, MoE recipe]  */
  int32_t top_k;          /* experts evaluated per row (1..min(E, 32)); ignored when E == 0 */
  int32_t w_dtype;        /* 0: projections in the model dtype; PLT_MXFP4: the four per-layer projections
                             (QKV, output, gate/up, down) on MXFP4 weights and MXFP8 activations, see
                             "Low-bit projections" below; in a mixture-of-experts model every expert's
                             gate/up and down matrices, the router staying in bf16 (needs dtype ==
                             PLT_BF16 and d_model, ffn_hidden, n_heads * head_dim multiples of 128) */
} plt_config;

typedef struct plt_model plt_model; /* opaque */
typedef struct plt_kv plt_kv;       /* opaque */

/* Tensors of the weight blob, in blob order:
 *   EMB [vocab, d]; per layer: NORM1 [d], WQKV [(Hq+2Hkv)*D, d] (rows: all Q heads, then all
 *   K heads, then all V heads), GATE_W [Hq, D], GATE_B [Hq], WO [d, Hq*D], NORM2 [d],
 *   WGU [2F, d] (rows: W_gate then W_up), WDOWN [d, F]; then NORM_F [d]; then HEAD [vocab, d]
 *   (absent when tie_embeddings).  Norm gains, gate weight and gate bias are always float;
 *   the other tensors have the model dtype.  Every tensor starts at a multiple of 256 bytes.
 *   Mixture-of-experts models (n_experts = E > 0): ROUTER [E, d] follows NORM2, and the expert
 *   matrices carry a leading expert axis: WGU [E, 2F, d] (per expert: its W_gate rows, then its
 *   W_up rows), WDOWN [E, d, F].  PLT_F32 keeps every expert matrix row-major; PLT_BF16 stores each
 *   expert matrix [N, K] strip by strip in matrix-core load order: element (n, k) of the matrix
 *   sits at element index plt_moe_weight_index(n, k, K) of that expert's N*K block (16-row strips;
 *   inside a strip 32-wide k chunks; inside a chunk [k/8 mod 4][n mod 16][k mod 8]), so that the
 *   grouped GEMM streams every strip as one contiguous run.
 *   Low-bit models (w_dtype = PLT_MXFP4): WQKV, WO, WGU, WDOWN hold e2m1 codes (element count N*K, two per
 *   byte) and each is followed by its scale tensor WQKV_SC, WO_SC, WGU_SC, WDOWN_SC (element count = bytes),
 *   both in the layouts plt_mx_quantize_weights writes; embedding, head, router and float tensors are
 *   unchanged.  With experts, WGU holds E matrices [2F, d] and WDOWN E matrices [d, F] back to back (expert e's
 *   codes start at e * N*K/2 bytes, its scales at e * plt_mx_weight_scale_bytes(N, K)). */
enum { PLT_W_EMB = 0, PLT_W_NORM1, PLT_W_WQKV, PLT_W_GATE_W, PLT_W_GATE_B, PLT_W_WO,
       PLT_W_NORM2, PLT_W_WGU, PLT_W_WDOWN, PLT_W_NORM_F, PLT_W_HEAD, PLT_W_ROUTER,
       PLT_W_WQKV_SC, PLT_W_WO_SC, PLT_W_WGU_SC, PLT_W_WDOWN_SC };

/* Total size of the weight blob in bytes (0 if the configuration is invalid). */
size_t plt_weights_bytes(const plt_config* cfg);

/* Byte offset and element count of one tensor inside the blob.  `layer` is ignored for EMB,
 * NORM_F and HEAD.  PLT_EINVAL for an invalid configuration / tensor id / layer. */
int plt_weights_offset(const plt_config* cfg, int32_t layer, int32_t which,
                       size_t* host_off_out, size_t* host_nelem_out);

/* Creates a model over a weight blob that already lies in device memory (layout above; the
 * blob must stay alive and unchanged while the model exists).  [Alg. 1 "Require"] */
int plt_init(const plt_config* cfg, const void* dev_weights, size_t nbytes, void* hip_stream,
             plt_model** out);
void plt_free(plt_model* m);

/* Bytes of device memory a KV object for `batch` sequences of up to max_ctx positions needs
 * (physical: positions are padded to multiples of 32, of 64 for e4m3 caches), and the logical size
 * 2 * layers * Hkv * D * (n_ctx + (L-1) * w) * sizeof(elem) * batch of Table 1 (row 5; row 2
 * in vanilla-loop and own-KV modes: 2 * layers * Hkv * D * L * n_ctx; row 4: ... * n_ctx). */
size_t plt_kv_bytes(const plt_model* m, int32_t batch, int32_t max_ctx);
size_t plt_kv_logical_bytes(const plt_model* m, int32_t batch, int32_t n_ctx);

/* Binds the cache layout to the caller's device buffer (>= plt_kv_bytes, 256-byte aligned),
 * clears it, and allocates the per-step activation scratch (the library's only hipMalloc besides
 * plt_init's small tables).  [Sec. 2.2.2: one shared cache + (L-1) windows] */
int plt_kv_alloc(plt_model* m, int32_t batch, int32_t max_ctx, void* dev_buf, size_t nbytes,
                 plt_kv** out);
void plt_kv_free(plt_kv* kv);

/* Prefill [Alg. 1 l.1-3 = Alg. 2 forward]: consumes dev_tokens [batch, n] (int32, row-major),
 * fills the shared cache for positions 0..n-1, the windows and the carried states, and
 * writes the greedy next token of every sequence to dev_next [batch] and, if not NULL, the
 * last position's logits to dev_logits [batch, vocab] (float).  Restarts the kv object.
 * Loop-major over the whole prompt, i.e. the sequential execution of the method (loop l of every
 * position before loop l + 1 of any), in chunks of whole sequences (about 16384 rows at a time).
 * dev_workspace: caller-owned device buffer (256-byte aligned) of at least
 * plt_prefill_workspace_bytes(m, kv, n) bytes for one chunk's activations; its contents are
 * undefined afterwards.  Asynchronous on the model's stream; PLT_ENOMEM if the workspace is too
 * small, PLT_ECTXFULL if n > max_ctx (no state change in either case). */
size_t plt_prefill_workspace_bytes(const plt_model* m, const plt_kv* kv, int32_t n);
int plt_prefill(plt_model* m, plt_kv* kv, const int32_t* dev_tokens, int32_t n,
                int32_t* dev_next, float* dev_logits, void* dev_workspace, size_t workspace_bytes);

/* One decode step [Alg. 1 l.5-9]: consumes the newest token of every sequence
 * (dev_tokens [batch]), runs the L loop stages of this position as one pass, appends to the
 * caches, updates the carried states and writes the next greedy token (and logits). */
int plt_decode_step(plt_model* m, plt_kv* kv, const int32_t* dev_tokens, int32_t* dev_next,
                    float* dev_logits);

/* Replay mode of plt_decode_step (off by default).  While on, a step is issued as ONE HIP graph launch: the
 * launch sequence of the step (about 220 dependent kernels for 24 layers) is recorded by stream capture the first
 * time and whenever dev_tokens / dev_next / dev_logits or the attention's split count change (the split count
 * depends on the context length only for batches that leave compute units idle), and replayed otherwise -- the
 * position is a device-side counter, so the same recorded launches serve every position [Alg. 1 l.5-9 is the same
 * work at every step].  The graph holds kernel nodes only (the step clears no memory).  Results are those of the
 * eager step bit for bit.  If capture or instantiation fails, nothing has been launched, the state is unchanged and
 * the step returns PLT_EHIP.  The stream handed to plt_init must not be the legacy NULL stream while this is on
 * (stream capture does not work on it).  Ignored while plt_profile_enable is on (events are recorded eagerly). */
int plt_use_graph(plt_model* m, int32_t on);

/* Number of positions consumed so far (prompt + decode steps), or a negative status. */
int32_t plt_kv_position(const plt_kv* kv);

const char* plt_last_error(void);

/* ---------------------------------------------------------------- test and bench hooks */

/* Sets the position counter without touching cache contents (bench: time steps at a fixed
 * context; tests: continue after plt_kv_import).  0 <= pos <= max_ctx. */
int plt_kv_set_position(plt_kv* kv, int32_t pos);

/* Copies one sequence's cache of one layer to / from host memory in a plain layout,
 * element type = the cache's (model dtype, or one e4m3 byte per element):
 *   shared K [Hkv, n, D], shared V [Hkv, n, D], then (CLP mode, L > 1) ring K
 *   [L-1, Hkv, w, D] and ring V [L-1, Hkv, w, D] in slot order (slot = position mod w).
 * `cache` selects the loop's cache in vanilla-loop and own-KV modes (0-based), must be 0 otherwise.
 * host_nbytes must equal plt_kv_export_bytes(kv, n). */
size_t plt_kv_export_bytes(const plt_kv* kv, int32_t n);
int plt_kv_export(plt_kv* kv, int32_t seq, int32_t layer, int32_t cache, int32_t n,
                  void* host_dst, size_t host_nbytes);
int plt_kv_import(plt_kv* kv, int32_t seq, int32_t layer, int32_t cache, int32_t n,
                  const void* host_src, size_t host_nbytes);

/* Timing-only aliasing of the shared caches (bench hook; results are meaningless while it is on): kv objects
 * created AFTER this call keep the shared K/V of only phys_layers layers in memory, and layer m streams and
 * appends to the memory of layer m mod phys_layers (windows stay per layer).  A batch whose shared cache exceeds
 * the device (256 sequences x 8192 positions x 24 layers = 412 GB in bf16) can then be timed at its real
 * per-layer shape: every layer still streams its full 17 GB, far more than any cache on the die holds, so
 * the bytes moved per step are the real ones.  phys_layers = 0 switches it off. */
int plt_kv_alias_layers(plt_model* m, int32_t phys_layers);

/* Carried states H^l[p-1], l = 1..L-1, of every sequence: float [batch, L-1, d]. */
int plt_get_carry(plt_kv* kv, float* host_dst, size_t host_nbytes);
int plt_set_carry(plt_kv* kv, const float* host_src, size_t host_nbytes);
/* Residual-stream rows after the last layer of the most recent decode step: float
 * [batch, L, d] (row l = loop l+1's output H^(l+1)[p]). */
int plt_get_hidden(plt_kv* kv, float* host_dst, size_t host_nbytes);
/* One layer of block f on the decode micro-batch from a GIVEN residual stream [Alg. 3 l.1-6, then the
 * feed-forward]: host_x_in float [batch, L, d] (row (b, l) = loop l+1 of sequence b) is taken as the input of
 * layer `layer` at the position the next plt_decode_step would consume; the layer runs exactly as inside that
 * step (its K/V for this position are appended to the shared cache / windows of that layer), and the layer's
 * output rows are returned in host_x_out.  The position counter does not move; the carried states and the
 * other layers' caches are untouched.  Lets a test feed every layer the reference's layer input (per-layer
 * teacher forcing), so that a single layer is compared at the stated tolerance without the accumulation of
 * roundings over depth.  CLP modes only; synchronises. */
int plt_debug_layer(plt_model* m, plt_kv* kv, int32_t layer, const float* host_x_in, float* host_x_out,
                    size_t host_nbytes);
/* Low-bit dense models (w_dtype = PLT_MXFP4, n_experts = 0): the quantised activations that entered the four
 * projections of the layer the LAST plt_debug_layer call ran [inference efficiency evaluation recipe; formats under
 * "Low-bit projections" below].  which = 0: input of the QKV projection (normed rows, K = d_model), 1: input of the
 * output projection (attention output, K = n_heads * head_dim), 2: input of the gate/up projection (normed rows,
 * K = d_model), 3: input of the down projection (SwiGLU product, K = ffn_hidden).  host_codes: e4m3 bytes
 * [batch * L, K] row-major; host_scales: [batch * L, 16 * ceil(K / 512)] scale bytes in the order of
 * plt_mx_act_scale_index.  A quantiser decides integers from floats, so two correct implementations may round
 * an element that sits on a rounding boundary to neighbouring codes; with the device's own codes in hand a test can
 * give the reference exactly the operands the device multiplied and compare the layer without that ambiguity.
 * PLT_ESTATE before the first plt_debug_layer call; synchronises. */
int plt_debug_act_codes(plt_kv* kv, int32_t which, uint8_t* host_codes, size_t codes_nbytes,
                        uint8_t* host_scales, size_t scales_nbytes);

/* Kernel-only fused decode attention [Alg. 3 l.2-5, Eq. 2; first-loop row: global only].
 * All pointers are device pointers, element type `dtype`, in the cache's native layout:
 *   q        [B, L, Hq, D]                       (already rotated)
 *   k_share  [B, Hkv, n_pad * D]                 n_pad = plt_attn_pad(dtype, n_alloc); PLT_F32: rows
 *                                                [n_pad, D]; PLT_BF16 / PLT_FP8_E4M3: tiles of 32 / 64
 *                                                positions in the kernel's matrix-core load order
 *                                                (written by plt_attn_pack_k; see below)
 *   v_share  [B, Hkv, n_pad * D]                 blocks of 32 positions; PLT_F32: [D, 32], position
 *                                                fastest; PLT_BF16 / PLT_FP8_E4M3: 16-byte chunks (8 / 16
 *                                                positions of one feature) ordered [D/16][chunk of
 *                                                positions][feature % 16] (written by plt_attn_pack_v)
 *   k_ring   [B, L-1, Hkv, w_pad * D]            w_pad = plt_attn_pad(dtype, w); layout as k_share
 *   v_ring   [B, L-1, Hkv, w_pad * D]            layout as v_share
 *   z        [B, L-1, Hq] float gate logits;  y [B, L, Hq, D] output
 * dtype PLT_FP8_E4M3: q and y are bf16, the four cache arrays hold e4m3 bytes.
 * n_ctx shared entries and n_ring (<= w) ring slots are valid for every sequence.
 * scratch: device buffer of plt_attn_scratch_bytes(...) bytes (split partials).
 * n_splits <= 0 lets the library choose.  Rows of loop 0 get the global branch only.
 * The L * (Hq / Hkv) query rows that share one (sequence, kv head) stream are served by ONE pass over its cache
 * bytes while they number at most 16 (the matrix-core tile's width: every named configuration: 2..16 rows); from 17
 * rows on each further group of 16 is a workgroup of its own that streams the same cache bytes again.
 * plt_attn_pad: positions are padded to a multiple of 32 (64 for PLT_FP8_E4M3);
 * plt_attn_pad32(n) = plt_attn_pad(PLT_BF16, n). */
int32_t plt_attn_pad32(int32_t n);
int32_t plt_attn_pad(int32_t dtype, int32_t n);
size_t plt_attn_scratch_bytes(int32_t B, int32_t L, int32_t Hq, int32_t Hkv, int32_t D);
int plt_attn_decode(int32_t dtype, int32_t B, int32_t L, int32_t Hq, int32_t Hkv, int32_t D,
                    int32_t n_alloc, int32_t n_ctx, int32_t w, int32_t n_ring,
                    const void* dev_q, const void* dev_k_share, const void* dev_v_share,
                    const void* dev_k_ring, const void* dev_v_ring, const float* dev_z,
                    void* dev_y, void* dev_scratch, size_t scratch_bytes, int32_t n_splits,
                    void* hip_stream);

/* plt_attn_decode for callers that cannot allocate device memory or pass a workspace of their own: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks,
 * kernels and results as plt_attn_decode (identical bits for the same n_splits), but the split partials
 * live in a device array the library itself holds (PLT_ATTN_STATIC_SCRATCH_BYTES per GPU, resident until the
 * process ends); this call allocates and frees nothing and synchronises nothing.  A shape whose partials for
 * the chosen number of splits (n_splits <= 0: the library's choice) do not fit the array is refused with
 * PLT_ENOMEM and nothing is launched: B * Hkv * ceil(L * Hq / Hkv / 16) streams need
 * (n_splits * (32 + 16 D) + 16 D) * 4 bytes each (kernel-only configuration B 32, 4 kv heads, D 128, 2 splits:
 * 3.1 MiB).  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams,
 * two threads) race on it and must be serialised by the caller; calls on different GPUs are independent. */
enum { PLT_ATTN_STATIC_SCRATCH_BYTES = 8 << 20 };
int plt_attn_decode_static(int32_t dtype, int32_t B, int32_t L, int32_t Hq, int32_t Hkv, int32_t D,
                           int32_t n_alloc, int32_t n_ctx, int32_t w, int32_t n_ring,
                           const void* dev_q, const void* dev_k_share, const void* dev_v_share,
                           const void* dev_k_ring, const void* dev_v_ring, const float* dev_z,
                           void* dev_y, int32_t n_splits, void* hip_stream);

/* Device-side layout conversion for the hook above: plain [S, n, D] (S independent streams,
 * e.g. B*Hkv) -> K layout [S, n_pad * D] (pad positions zeroed) and V layout [S, n_pad * D] (see v_share above).
 * K layout of the 2-byte and 1-byte types: a tile of T = 32 (64) positions is T*D elements stored as
 * [a][kk][m][g][c] with c = 16 bytes' worth of consecutive features (8 / 16), m in 0..15, g in 0..3,
 * kk in 0..D/(4c)-1, a in 0..T/16-1; the element is position 2T/8*(m>>2) + (m&3) + 4a of the tile
 * (i.e. 8*(m>>2) + (m&3) + 4a, resp. 16*(m>>2) + (m&3) + 4a), feature kk*4c + g*c + its index in c:
 * one wavefront load of the attention kernel (lane = 16g + m reads piece 4m + g) is then one contiguous KiB,
 * and the 4c features of one key in chunk kk are 64 adjacent bytes.
 * Elements are moved, never converted: for PLT_FP8_E4M3 source and destination hold e4m3 bytes. */
/* Host-side statement of the K layout above: element index of (position pos, feature f) inside one
 * stream of head size D (no device work; -1 for a bad argument).  The append, pack and attention
 * kernels use the same function. */
int64_t plt_attn_k_index(int32_t dtype, int32_t pos, int32_t f, int32_t D);
/* The same for the V layout (v_share above): element index of (position pos, feature d) inside one stream.
 * PLT_F32: blocks of 32 positions stored [D][32].  PLT_BF16 / PLT_FP8_E4M3: a block's 16-byte chunks
 * (c = 8 / 16 consecutive positions of one feature) in the order [d / 16][position chunk][d % 16]: the 64
 * chunks of 16 features x 32 positions are one contiguous KiB (one wavefront load of the attention kernel),
 * and the chunks that one appended position touches lie 16 in a row. */
int64_t plt_attn_v_index(int32_t dtype, int32_t pos, int32_t d, int32_t D);
int plt_attn_pack_k(int32_t dtype, int32_t S, int32_t n, int32_t D, const void* dev_src,
                    void* dev_dst, void* hip_stream);
int plt_attn_pack_v(int32_t dtype, int32_t S, int32_t n, int32_t D, const void* dev_src,
                    void* dev_dst, void* hip_stream);

/* Kernel-only dense contraction used by every projection [Alg. 3 l.1 and l.6; FFN; head]:
 * c [M, N] (float) = a [M, K] * w [N, K]^T with a and w of type `dtype`, float accumulation. */
int plt_gemm(int32_t dtype, int32_t M, int32_t N, int32_t K, const void* dev_a,
             const void* dev_w, float* dev_c, void* dev_scratch, size_t scratch_bytes,
             void* hip_stream);
size_t plt_gemm_scratch_bytes(int32_t M, int32_t N, int32_t K);
/* Kernel-only form of the prefill's output / down projection, whose epilogue adds the product to the residual
 * stream [block f's two residual connections around Alg. 3 l.6 and the feed-forward]: x [M, N] (float, device,
 * updated in place) += a [M, K] * w [N, K]^T with bf16 a and w (device), float accumulation.  Only for the row counts
 * that take the 256 x 256 tile kernel (M >= 512, at least 200 tiles, K a multiple of 64); any other shape returns
 * PLT_EINVAL and leaves x untouched (the model adds those products in its residual + norm kernel instead). */
int plt_gemm_residual(int32_t M, int32_t N, int32_t K, const void* dev_a, const void* dev_w, float* dev_x,
                      void* hip_stream);

/* Kernel-only mixture-of-experts feed-forward [appendix, "MoE Models Recipe"; router reading in the
 * header comment]: for R rows a [R, d] (already normed), router [E, d], wgu [E, 2F, d], wdown [E, d, F]
 * (all of type `dtype`, device memory; PLT_BF16: the expert matrices in the strip order of
 * plt_moe_weight_index, as in the weight blob) writes
 *   y [R, d] float       = sum over the k selected experts e of p_e * W_down^e (silu(W_gate^e a) * W_up^e a)
 *   sel_e [R, k] int32   the selected experts in order of decreasing probability
 *   sel_p [R, k] float   their softmax probabilities
 * PLT_BF16 needs d % 64 == 0 and F % 64 == 0; E <= 256, k <= min(E, 32).  dev_scratch: device buffer of
 * plt_moe_scratch_bytes(...) bytes (index lists, the experts' hidden activations, k output slabs). */
int64_t plt_moe_weight_index(int32_t n, int32_t k, int32_t K); /* host only; -1 for a bad argument */
size_t plt_moe_scratch_bytes(int32_t dtype, int32_t R, int32_t d, int32_t F, int32_t E, int32_t k);
int plt_moe_ffn(int32_t dtype, int32_t R, int32_t d, int32_t F, int32_t E, int32_t k, const void* dev_a,
                const void* dev_router, const void* dev_wgu, const void* dev_wdown, float* dev_y,
                int32_t* dev_sel_e, float* dev_sel_p, void* dev_scratch, size_t scratch_bytes,
                void* hip_stream);

/* Low-bit projections [inference efficiency evaluation recipe: "W4A8 quantization of linear layers"; the
 * paper names no format].  Reading taken: the OCP microscaling formats, which gfx950's block-scaled
 * matrix-core instruction consumes directly.  A tensor is cut into blocks of 32 consecutive elements along
 * the contraction axis k; a block stores one scale byte s (the power of two 2^(s - 127), with
 * s - 127 = floor(log2(max |v|)) - emax, clamped to -127..127; an all-zero block stores 0) and 32 elements
 * v / 2^(s - 127) rounded to the element format, nearest even, saturating:
 *   weights      e2m1, 4 bits (magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6; emax 2), two per byte, even k low nibble
 *   activations  e4m3, 8 bits (the cache format above; emax 8)
 * Layouts (all device memory, N % 16 == 0, K % 128 == 0):
 *   weight codes  [N/16 strips][K/128 chunks][64 lanes][16 bytes]: lane 16 g + m of a chunk holds row m of
 *                 the strip, k = 32 g .. 32 g + 31 of the chunk; plt_mx_weight_code_index(n, k, K) is the byte
 *   weight scales [N/16][ceil(K/512)][64 lanes][4]: plt_mx_weight_scale_index(n, b, K) is the byte of row n,
 *                 k block b; bytes of chunks beyond K are 0
 *   act codes     row-major [M][K]
 *   act scales    [M][16 * ceil(K/512)]: the byte of k block b of a row is plt_mx_act_scale_index(b)
 *                 = 16 (b / 16) + 4 (b mod 4) + (b / 4) mod 4; bytes of blocks beyond K are 0
 * plt_mx_quantize_weights: bf16 [N, K] row-major -> codes + scales.  plt_mx_quantize_act: float or bf16
 * [M, K] (K % 32 == 0) -> codes + scales.  plt_gemm_mx: c [M, N] float = the exact product of the two
 * dequantised operands, float accumulation; dev_scratch of plt_gemm_mx_scratch_bytes bytes (K-range slabs).
 * The index functions run on the host; they return -1 for a bad argument. */
size_t plt_mx_weight_code_bytes(int32_t N, int32_t K);
size_t plt_mx_weight_scale_bytes(int32_t N, int32_t K);
size_t plt_mx_act_scale_bytes(int32_t M, int32_t K);
int64_t plt_mx_weight_code_index(int32_t n, int32_t k, int32_t K);
int64_t plt_mx_weight_scale_index(int32_t n, int32_t b, int32_t K);
int32_t plt_mx_act_scale_index(int32_t b);
int plt_mx_quantize_weights(int32_t N, int32_t K, const void* dev_src_bf16, void* dev_codes, void* dev_scales,
                            void* hip_stream);
int plt_mx_quantize_act(int32_t dtype, int32_t M, int32_t K, const void* dev_src, void* dev_codes,
                        void* dev_scales, void* hip_stream);
size_t plt_gemm_mx_scratch_bytes(int32_t M, int32_t N, int32_t K);
int plt_gemm_mx(int32_t M, int32_t N, int32_t K, const void* dev_a_codes, const void* dev_a_scales,
                const void* dev_w_codes, const void* dev_w_scales, float* dev_c, void* dev_scratch,
                size_t scratch_bytes, void* hip_stream);
/* The gate/up projection of the low-bit feed-forward block with its activation and the quantiser of the
 * down projection's operand [inference efficiency evaluation recipe; SwiGLU feed-forward of the backbone]:
 * h[M, F] = silu(a Wg^T) * (a Wu^T) from the low-bit operands above, w = [gate rows; up rows] = [2F, K]
 * (F % 32 == 0, K % 128 == 0), written as e4m3 codes [M][F] and block scales [M][16 * ceil(F/512)] in the
 * activation layout (bytes of blocks beyond F are 0).  For decode-sized M and F >= 4096 one kernel (the
 * activation and the quantiser are the product's epilogue); otherwise the product's K-range slabs go through
 * dev_scratch (plt_gemm_mx_swiglu_scratch_bytes) and a second kernel.  The result must not alias the operand.
 * All pointers device memory, 16-byte aligned; PLT_EINVAL / PLT_ENOMEM as for plt_gemm_mx. */
size_t plt_gemm_mx_swiglu_scratch_bytes(int32_t M, int32_t F, int32_t K);
int plt_gemm_mx_swiglu(int32_t M, int32_t F, int32_t K, const void* dev_a_codes, const void* dev_a_scales,
                       const void* dev_w_codes, const void* dev_w_scales, void* dev_h_codes, void* dev_h_scales,
                       void* dev_scratch, size_t scratch_bytes, void* hip_stream);

/* Plain device-to-device copy kernel (16 bytes per lane): the known-size reference for HBM
 * traffic counters and a practical bandwidth ceiling.  nbytes and both pointers must be
 * multiples of 16; the buffers must not overlap. */
int plt_stream_copy(void* dev_dst, const void* dev_src, size_t nbytes, void* hip_stream);
/* Read-only counterpart (a practical ceiling for a pure read stream such as decode attention):
 * reads nbytes (a multiple of 32 KiB) and writes one word per thread to dev_out (>= 2 MiB). */
int plt_stream_read(const void* dev_src, size_t nbytes, void* dev_out, size_t out_bytes, void* hip_stream);

/* Bench instrumentation.  `mask` selects launch classes (bit 1 << PLT_PROF_ATTN: the fused
 * attention kernel; bit 1 << PLT_PROF_GEMM: every projection GEMM; 0 = off).  While selected, every
 * such launch made by plt_decode_step is bracketed by a pair of hipEvents recorded on the model's
 * stream.  plt_profile_read synchronises the
 * stream, returns the summed elapsed milliseconds and the number of launches of one class
 * since the last reset, and optionally resets the counters. */
enum { PLT_PROF_ATTN = 0, PLT_PROF_GEMM = 1 };
int plt_profile_enable(plt_model* m, int32_t mask);
int plt_profile_read(plt_model* m, int32_t klass, double* host_ms_sum, int64_t* host_launches,
                     int32_t reset);

#ifdef __cplusplus
}
#endif
#endif /* PLT_H_ */
