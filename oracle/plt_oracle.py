"""CPU oracle for the Parallel Loop Transformer (PLT) forward / decode path.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, float64 statement of what the
HIP library must compute.  Only tests, the smoke check and the bench's cpu_baseline leg may
import it; the product path never does.  It shares no code with the HIP path and imports
nothing from it.

Every function cites the passage of the paper (arxiv 2510.24824) it follows:

  Eq. (1)   vanilla loop transformer            -> PLTOracle.vanilla_loop_forward
  Alg. 1    PLT decoding (cross-loop parallel)  -> PLTOracle.clp_prefill / clp_decode_step
  Alg. 2    PLT training-time forward           -> PLTOracle.seq_forward
  Alg. 3    non-first-loop attention            -> gated_attention_row / decode_attention
  Eq. (2)   sigmoid gate merge                  -> gate_merge
  Sec. 2.2.2  first-loop KV sharing, window of the most recent w entries -> RingKV
  Table 1 rows 3 and 4 (ablations: CLP with per-loop KV; CLP + KV share without the window) -> variant=
  Appendix, "MoE Models Recipe" (SwiGLU experts, k of E experts per token)              -> moe_route / moe_ffn
  Inference efficiency evaluation recipe ("W4A8 quantization of linear layers")         -> mx_quantize / mx_linear

Where the paper is silent the following readings are taken (each also listed in the
design notes of the repository):
  * block f = pre-norm decoder layer: RMSNorm -> attention -> residual, RMSNorm -> SwiGLU -> residual
  * rotary position embedding (rotate-half pairing, angle from the absolute position p)
    on Q and on every cached K; softmax scale 1/sqrt(D) in both branches
  * the state carried between loops is the residual stream after the last layer (before
    the final norm); the final norm feeds only the classifier head
  * the global branch of a non-first loop at position p sees shared keys 0..p inclusive
  * the window holds positions max(0, p-w+1)..p (w entries including the current one)
  * the gate logit of head h is <q_h, wg_h> + bg_h on q as produced by f_qkv (before RoPE),
    one scalar per head; g multiplies the LOCAL branch (Eq. 2)
  * one weight set serves every loop; query head h reads kv head h // (H_q / H_kv)
  * argmax ties resolve to the lowest index
  * mixture-of-experts feed-forward (n_experts > 0; the paper names only "SwiGLU experts" and "8 in 64" and
    builds on OLMoE, whose router is the one taken here): router logits r = W_r b on the normed
    row b, p = softmax(r) over all E experts, the k experts with the largest p are evaluated
    (equal p: lowest index first) and their outputs are summed with weights p_e as they are --
    the k selected probabilities are NOT renormalised to sum to one; no shared expert, no bias

  * low-bit linear layers (w_mx=True).  The paper serves its models with 4-bit weights and 8-bit
    activations in the linear layers and names no format.  Reading taken: the OCP microscaling
    formats.  A tensor is cut into blocks of 32 consecutive elements along the contraction axis; a
    block stores a shared power-of-two scale X = 2^(floor(log2(max |v|)) - emax) (emax = largest
    exponent of the element format; an all-zero block: 2^-127) and 32 elements v / X rounded to the
    element format, nearest even, saturating.  Weights: element format e2m1 (values 0, 0.5, 1, 1.5, 2,
    3, 4, 6 and their negatives; emax 2), quantised once from the bf16 weights.  Activations: element
    format e4m3 (emax 8), quantised where they enter a projection (the normed rows, the attention
    output, the SwiGLU product).  A projection is the exact product of the two dequantised operands.
    The four per-layer projections (QKV, output, gate/up, down) are quantised -- in a mixture-of-experts
    model every expert's gate, up and down matrices, while the router matrix keeps its precision and reads the
    quantised normed row; embedding, classifier head, norms, gate vector and every other operation keep
    their precision.

Precision: float64 everywhere.  With kv_bf16=True the K and V entries are rounded to
bfloat16 when they are stored (the device keeps its caches in bfloat16), nothing else is.
With kv_fp8=True they are instead rounded to the 8-bit float format e4m3 (4 exponent bits, 3
mantissa bits, no infinities, largest value 448; the OCP "e4m3fn" format) with saturation: the
paper serves its models with FP8 self-attention [inference efficiency evaluation recipe]; the
reading taken here is an FP8 *storage* format for every cached K and V (after RoPE, unit scale),
while queries, softmax weights and all sums keep full precision.
Parity status: every function here is pinned by tests/test_oracle_pins.py, test_oracle_moe_pins.py
and test_oracle_mx_pins.py.
"""
from __future__ import annotations

import math
import numpy as np

__all__ = ["OracleShape", "PLTOracle", "rmsnorm", "rope", "softmax_attend", "gate_merge",
           "gated_attention_row", "decode_attention", "kv_cache_bytes", "bf16_round", "e4m3_round",
           "swiglu_ffn", "moe_route", "moe_ffn", "e2m1_round", "mx_quantize", "mx_dequantize", "mx_linear"]


# ----------------------------------------------------------------------------- helpers

def bf16_round(x: np.ndarray) -> np.ndarray:
    """Nearest-even rounding of float values to bfloat16 (8-bit exponent, 7-bit mantissa)."""
    f = np.asarray(x, dtype=np.float32)
    bits = f.view(np.uint32).astype(np.int64)
    keep_odd = (bits >> 16) & 1
    bits = ((bits + 0x7FFF + keep_odd) >> 16) << 16
    return bits.astype(np.uint32).view(np.float32).astype(np.float64)


def e4m3_round(x: np.ndarray) -> np.ndarray:
    """Nearest-even rounding to the 8-bit float e4m3 (OCP e4m3fn), saturating at +-448.

    Format: 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits; normal values
    2^(e-7) * (1 + m/8) for e = 1..15 (e = 15, m = 7 is NaN, so the largest is 1.75 * 2^8 = 448);
    subnormals m/8 * 2^-6.  Neighbouring values in the binade [2^E, 2^(E+1)) are 2^(E-3) apart,
    and 2^-9 apart below 2^-6."""
    a = np.clip(np.asarray(x, np.float64), -448.0, 448.0)
    mag = np.abs(a)
    _, ex = np.frexp(mag)                       # mag = f * 2^ex with f in [0.5, 1)
    E = np.maximum(ex - 1, -6)                  # binade of mag, clamped to the subnormal range
    step = np.ldexp(1.0, E - 3)
    return np.sign(a) * np.rint(mag / step) * step      # rint: ties to even


def e2m1_round(x: np.ndarray) -> np.ndarray:
    """Nearest-even rounding to the 4-bit float e2m1 (1 sign, 2 exponent bits with bias 1, 1 mantissa bit):
    magnitudes 0, 0.5 (subnormal), 1, 1.5, 2, 3, 4, 6; saturating at +-6.  Neighbours are 0.5 apart below 2,
    1 apart in [2, 4) and 2 apart in [4, 8)."""
    a = np.clip(np.asarray(x, np.float64), -6.0, 6.0)
    mag = np.abs(a)
    _, ex = np.frexp(mag)
    E = np.maximum(ex - 1, 0)                   # binade of mag; everything below 1 shares the subnormal step
    step = np.ldexp(1.0, E - 1)
    return np.sign(a) * np.minimum(np.rint(mag / step) * step, 6.0)     # rint: ties to even


MX_BLOCK = 32
_MX_FORMATS = {"e2m1": (2, e2m1_round), "e4m3": (8, e4m3_round)}      # element format -> (emax, rounding)


def mx_quantize(x: np.ndarray, fmt: str):
    """Microscaling quantisation of x[..., K] (K a multiple of 32) along the last axis.

    Returns (q, e): q[..., K] the element values (on the element format's grid, float64) and
    e[..., K/32] the integer scale exponents, so that the represented tensor is q * 2^e per block.
    e = floor(log2(max |block|)) - emax, clamped to [-127, 127]; an all-zero block gets -127."""
    emax, rnd = _MX_FORMATS[fmt]
    x = np.asarray(x, np.float64)
    K = x.shape[-1]
    assert K % MX_BLOCK == 0
    blk = x.reshape(*x.shape[:-1], K // MX_BLOCK, MX_BLOCK)
    amax = np.max(np.abs(blk), axis=-1)
    _, ex = np.frexp(amax)                      # amax = f * 2^ex, f in [0.5, 1): floor(log2(amax)) = ex - 1
    e = np.where(amax > 0, np.clip(ex - 1 - emax, -127, 127), -127).astype(np.int64)
    q = rnd(blk * np.ldexp(1.0, -e)[..., None])
    return q.reshape(x.shape), e


def mx_dequantize(q: np.ndarray, e: np.ndarray) -> np.ndarray:
    q = np.asarray(q, np.float64)
    blk = q.reshape(*q.shape[:-1], q.shape[-1] // MX_BLOCK, MX_BLOCK)
    return (blk * np.ldexp(1.0, np.asarray(e))[..., None]).reshape(q.shape)


def mx_linear(a: np.ndarray, w_q: np.ndarray, w_e: np.ndarray) -> np.ndarray:
    """y = W_dq a_dq for one row a[K]: a is quantised to e4m3 blocks here, W [N, K] arrives quantised
    (e2m1 element values w_q and block exponents w_e [N, K/32])."""
    a_q, a_e = mx_quantize(a, "e4m3")
    return mx_dequantize(w_q, w_e) @ mx_dequantize(a_q, a_e)


class OracleShape:
    def __init__(self, n_layers, d_model, n_heads, n_kv_heads, head_dim, ffn_hidden, vocab,
                 n_loops, window, rope_theta=10000.0, norm_eps=1e-5, tie_embeddings=True,
                 n_experts=0, top_k=0):
        self.n_layers, self.d_model = int(n_layers), int(d_model)
        self.n_heads, self.n_kv_heads, self.head_dim = int(n_heads), int(n_kv_heads), int(head_dim)
        self.ffn_hidden, self.vocab = int(ffn_hidden), int(vocab)
        self.n_loops, self.window = int(n_loops), int(window)
        self.rope_theta, self.norm_eps = float(rope_theta), float(norm_eps)
        self.tie_embeddings = bool(tie_embeddings)
        # n_experts = 0: dense SwiGLU feed-forward; > 0: ffn_hidden is the hidden size of each expert
        self.n_experts, self.top_k = int(n_experts), int(top_k)
        assert self.n_experts == 0 or 1 <= self.top_k <= self.n_experts
        assert self.n_heads % self.n_kv_heads == 0 and self.head_dim % 2 == 0


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x * gain / sqrt(mean(x^2) + eps) over the last axis (reading: pre-norm RMSNorm)."""
    x = np.asarray(x, np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, np.float64)


def rope(x: np.ndarray, p: int, theta: float) -> np.ndarray:
    """Rotary embedding of x[..., D] at absolute position p; dim j pairs with j + D/2."""
    x = np.asarray(x, np.float64)
    D = x.shape[-1]
    half = D // 2
    j = np.arange(half, dtype=np.float64)
    ang = p * theta ** (-2.0 * j / D)
    c, s = np.cos(ang), np.sin(ang)
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def softmax_attend(q: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """sum_j softmax_j(<q, K[j]> / sqrt(D)) V[j] for one query q[D], K[n,D], V[n,D].

    Alg. 3 lines 2 and 3 each are one call of this (global: all shared entries; local:
    the window's entries).
    """
    q = np.asarray(q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    s = K @ q / math.sqrt(q.shape[-1])
    s = s - np.max(s)
    e = np.exp(s)
    return (e / np.sum(e)) @ V


def gate_merge(y_local: np.ndarray, y_global: np.ndarray, z: float) -> np.ndarray:
    """Eq. (2): g = sigmoid(z);  y = g * y_local + (1 - g) * y_global."""
    g = 1.0 / (1.0 + math.exp(-float(z)))
    return g * np.asarray(y_local, np.float64) + (1.0 - g) * np.asarray(y_global, np.float64)


def gated_attention_row(q, K_share, V_share, K_loc, V_loc, z) -> np.ndarray:
    """Alg. 3 lines 2-5 for one query head of a non-first loop."""
    y_glob = softmax_attend(q, K_share, V_share)
    y_loc = softmax_attend(q, K_loc, V_loc)
    return gate_merge(y_loc, y_glob, z)


def decode_attention(q, k_share, v_share, k_ring, v_ring, z, n_ctx=None, n_ring=None):
    """Fused decode attention of one CLP step, all sequences (kernel-only configuration).

    q [B,L,Hq,D]; k_share, v_share [B,Hkv,N,D]; k_ring, v_ring [B,L-1,Hkv,w,D] in slot
    order; z [B,L-1,Hq] gate logits.  n_ctx (<= N) shared entries and n_ring (<= w) ring
    slots are valid (default: all).  Row l = 0 is the first loop: global attention only
    (first loop == plain transformer).  Rows l >= 1: Alg. 3 lines 2-5.  Returns y [B,L,Hq,D].
    """
    q = np.asarray(q, np.float64)
    B, L, Hq, D = q.shape
    Hkv = k_share.shape[1]
    G = Hq // Hkv
    n_ctx = k_share.shape[2] if n_ctx is None else int(n_ctx)
    y = np.zeros((B, L, Hq, D), np.float64)
    for b in range(B):
        for h in range(Hq):
            kh = h // G
            Ks = np.asarray(k_share[b, kh, :n_ctx], np.float64)
            Vs = np.asarray(v_share[b, kh, :n_ctx], np.float64)
            y[b, 0, h] = softmax_attend(q[b, 0, h], Ks, Vs)
            for l in range(1, L):
                nr = k_ring.shape[3] if n_ring is None else int(n_ring)
                y[b, l, h] = gated_attention_row(q[b, l, h], Ks, Vs,
                                                 k_ring[b, l - 1, kh, :nr], v_ring[b, l - 1, kh, :nr],
                                                 z[b, l - 1, h])
    return y


def swiglu_ffn(b, w_gate, w_up, w_down, hidden_in=None) -> np.ndarray:
    """W_down (silu(W_gate b) * (W_up b)) for one row b[d]; matrices are [out, in].  hidden_in, if given, is
    applied to the hidden vector before the down projection (low-bit models: its e4m3 block quantiser)."""
    b = np.asarray(b, np.float64)
    gte = np.asarray(w_gate, np.float64) @ b
    up = np.asarray(w_up, np.float64) @ b
    h = gte / (1.0 + np.exp(-gte)) * up
    return np.asarray(w_down, np.float64) @ (h if hidden_in is None else hidden_in(h))


def moe_route(b, router, top_k):
    """Router of the mixture-of-experts feed-forward for one row b[d], router [E, d].

    p = softmax(router b) over all E experts; returns (ids, p[ids], margin): the top_k experts
    in order of decreasing p (equal p: lowest index first), their probabilities (not
    renormalised) and the logit gap between the last selected and the best rejected expert
    (inf when top_k == E) -- tests use the gap to tell decisions that rounding could flip."""
    r = np.asarray(router, np.float64) @ np.asarray(b, np.float64)
    e = np.exp(r - np.max(r))
    p = e / np.sum(e)
    order = np.argsort(-p, kind="stable")
    ids = order[:top_k]
    margin = float(r[order[top_k - 1]] - r[order[top_k]]) if top_k < len(r) else math.inf
    return ids, p[ids], margin


def moe_ffn(b, W, top_k, margins=None, hidden_in=None) -> np.ndarray:
    """sum over the selected experts e of p_e * SwiGLU_e(b) [appendix, MoE models recipe; router
    reading in the header].  W: "router" [E, d], "w_gate" / "w_up" [E, F, d], "w_down" [E, d, F]."""
    ids, p, margin = moe_route(b, W["router"], top_k)
    if margins is not None:
        margins.append(margin)
    out = np.zeros(np.asarray(W["w_down"]).shape[1], np.float64)
    for e, pe in zip(ids, p):
        out += pe * swiglu_ffn(b, W["w_gate"][e], W["w_up"][e], W["w_down"][e], hidden_in)
    return out


def kv_cache_bytes(shape: OracleShape, n_ctx: int, elem_bytes: int, n_loops: int | None = None,
                   shared: bool = True) -> int:
    """Table 1, KV-cache column, as exact entry counts.

    PLT (shared=True): one global cache of n_ctx entries plus (L-1) windows of w entries,
    per layer, K and V.  Vanilla loop (shared=False): L full caches.
    """
    L = shape.n_loops if n_loops is None else n_loops
    per_entry = 2 * shape.n_layers * shape.n_kv_heads * shape.head_dim * elem_bytes
    if shared:
        return per_entry * (n_ctx + (L - 1) * shape.window)
    return per_entry * L * n_ctx


# ----------------------------------------------------------------------------- KV stores

class FullHistoryKV:
    """Keeps every K/V ever produced; the window is cut out by position.  Used by Alg. 2."""

    def __init__(self, store):
        self._store = store
        self.glob = {}   # (cache_id, layer) -> ([k...], [v...])
        self.loc = {}    # (loop, layer)     -> ([k...], [v...])

    def put_global(self, cache_id, m, p, k, v):
        ks, vs = self.glob.setdefault((cache_id, m), ([], []))
        assert len(ks) == p
        ks.append(self._store(k)); vs.append(self._store(v))

    def get_global(self, cache_id, m, p):
        ks, vs = self.glob[(cache_id, m)]
        return np.stack(ks[:p + 1]), np.stack(vs[:p + 1])

    def put_local(self, l, m, p, k, v, w):
        ks, vs = self.loc.setdefault((l, m), ([], []))
        assert len(ks) == p
        ks.append(self._store(k)); vs.append(self._store(v))

    def get_local(self, l, m, p, w):
        ks, vs = self.loc[(l, m)]
        lo = max(0, p - w + 1)
        return np.stack(ks[lo:p + 1]), np.stack(vs[lo:p + 1])


class RingKV:
    """The decoding-time cache of Sec. 2.2.2: one shared cache plus, for every non-first
    loop and layer, only the w most recent entries (slot = p mod w).  Used by Alg. 1."""

    def __init__(self, store, shape: OracleShape, max_ctx: int):
        self._store = store
        s = shape
        self.w = s.window
        self.ks = np.zeros((s.n_layers, max_ctx, s.n_kv_heads, s.head_dim))
        self.vs = np.zeros_like(self.ks)
        nl = max(s.n_loops - 1, 0)
        self.kr = np.zeros((nl, s.n_layers, s.window, s.n_kv_heads, s.head_dim))
        self.vr = np.zeros_like(self.kr)

    def _cache(self, cache_id):
        if cache_id == 1:
            return self.ks, self.vs
        if not hasattr(self, "extra"):
            self.extra = {}
        if cache_id not in self.extra:                # own-KV variant: one more full cache per loop
            self.extra[cache_id] = (np.zeros_like(self.ks), np.zeros_like(self.vs))
        return self.extra[cache_id]

    def put_global(self, cache_id, m, p, k, v):
        ks, vs = self._cache(cache_id)
        ks[m, p] = self._store(k); vs[m, p] = self._store(v)

    def get_global(self, cache_id, m, p):
        ks, vs = self._cache(cache_id)
        return ks[m, :p + 1], vs[m, :p + 1]

    def put_local(self, l, m, p, k, v, w):
        self.kr[l - 2, m, p % w] = self._store(k); self.vr[l - 2, m, p % w] = self._store(v)

    def get_local(self, l, m, p, w):
        n = min(p + 1, w)          # slots 0..n-1 are the valid ones, in slot (not time) order
        return self.kr[l - 2, m, :n], self.vr[l - 2, m, :n]

    def n_bytes(self, n_ctx: int, elem_bytes: int) -> int:
        per = self.ks.shape[2] * self.ks.shape[3] * elem_bytes
        return 2 * per * (self.ks.shape[0] * n_ctx + self.kr.shape[0] * self.kr.shape[1] * self.kr.shape[2])


# ----------------------------------------------------------------------------- the model

class PLTOracle:
    """One sequence at a time (sequences of a batch never interact)."""

    def __init__(self, shape: OracleShape, weights: dict, kv_bf16: bool = False, variant: str = "plt",
                 kv_fp8: bool = False, w_mx: bool = False):
        """variant selects the row of Table 1 that is computed (all share the cross-loop shift):
          "plt"            row 5: shared first-loop KV + gated sliding window (the method)
          "clp_share_only" row 4: non-first loops attend the shared first-loop KV only (no own K/V, no gate)
          "clp_own_kv"     row 3: every loop keeps and attends its own full KV cache (no sharing, no gate)"""
        assert variant in ("plt", "clp_share_only", "clp_own_kv")
        self.variant = variant
        self.s = shape
        self.w = weights
        assert not (kv_bf16 and kv_fp8)
        self.kv_bf16, self.kv_fp8 = kv_bf16, kv_fp8
        self._store = bf16_round if kv_bf16 else e4m3_round if kv_fp8 else (lambda a: np.asarray(a, np.float64))
        self._head = weights["emb"] if shape.tie_embeddings else weights["head"]
        self.route_margins = []     # logit gap of every routing decision taken (MoE models)
        # bookkeeping for per-layer comparisons: when set to a list, every layer evaluated by f() appends
        # (loop l, layer m, position p, the layer's input row, the layer's output row); no arithmetic depends on it
        self.layer_trace = None
        # low-bit models, for tests that must not depend on which way a value on a rounding boundary falls: when
        # act_trace is a list, every value about to be block-quantised is appended as (loop l, layer m, stage, value)
        # with stage 0 = QKV input, 1 = output-projection input, 2 = gate/up input, 3 = down-projection input; and when
        # act_override maps (l, m, stage) to a vector, that vector is used IN PLACE of this oracle's own quantised
        # value (e.g. the dequantised codes another implementation chose).  Neither changes any arithmetic by itself.
        self.act_trace = None
        self.act_override = None
        # low-bit linear layers: the four projections of every layer on microscaling operands
        self.w_mx = w_mx
        if w_mx:
            self.wq_mx = []             # (expert matrices: blocks run along the last axis as well; the router keeps its precision)
            for W in weights["layers"]:
                self.wq_mx.append({name: mx_dequantize(*mx_quantize(W[name], "e2m1"))
                                   for name in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")})

    # -- block f: one pass of the whole layer stack for one row at position p in loop l (1-based)
    def f(self, x, p, l, kv, global_cache_id=1, plain=False, layers=None):
        """Transformer stack applied to one hidden row.

        l == 1 (or plain=True): ordinary causal attention; its rotated K and its V are
        appended to global cache `global_cache_id` (the first loop's cache is the shared one).
        l >= 2: Alg. 3 -- global attention over the shared cache (0..p inclusive), sliding
        window attention over this loop's own last w entries, Eq. (2) gate merge.
        layers: the layers to apply (default: all, in order); tests apply one layer to a given row.
        """
        s = self.s
        Hq, Hkv, D = s.n_heads, s.n_kv_heads, s.head_dim
        G = Hq // Hkv
        x = np.asarray(x, np.float64).copy()
        first = plain or l == 1
        share_only = False
        if not plain and l >= 2:
            if self.variant == "clp_own_kv":          # Table 1 row 3: loop l on its own cache l
                first, global_cache_id = True, l
            elif self.variant == "clp_share_only":    # Table 1 row 4: global branch only
                share_only = True
        for m in (range(s.n_layers) if layers is None else layers):
            W = self.w["layers"][m]
            x_in = x
            a = rmsnorm(x, W["norm1"], s.norm_eps)
            act_in = (lambda t, stage: t)
            if self.w_mx:                       # quantised projections: dequantised weights, e4m3-block inputs
                W = {**W, **self.wq_mx[m]}

                def act_in(t, stage, m=m):
                    if self.act_trace is not None:
                        self.act_trace.append((l, m, stage, np.array(t, np.float64)))
                    if self.act_override is not None and (l, m, stage) in self.act_override:
                        return np.asarray(self.act_override[(l, m, stage)], np.float64)
                    return mx_dequantize(*mx_quantize(t, "e4m3"))
            a = act_in(a, 0)
            q = (np.asarray(W["wq"], np.float64) @ a).reshape(Hq, D)          # Alg. 3 l.1
            k = (np.asarray(W["wk"], np.float64) @ a).reshape(Hkv, D)
            v = (np.asarray(W["wv"], np.float64) @ a).reshape(Hkv, D)
            if not first and not share_only:                                     # Alg. 3 l.4
                z = np.sum(q * np.asarray(W["gate_w"], np.float64), axis=-1) + np.asarray(W["gate_b"], np.float64)
            qr = rope(q, p, s.rope_theta)
            kr = rope(k, p, s.rope_theta)
            if first:
                kv.put_global(global_cache_id, m, p, kr, v)
            elif not share_only:
                kv.put_local(l, m, p, kr, v, s.window)
            Kg, Vg = kv.get_global(global_cache_id, m, p)                        # [p+1, Hkv, D]
            y = np.zeros((Hq, D))
            if first or share_only:
                for h in range(Hq):
                    y[h] = softmax_attend(qr[h], Kg[:, h // G], Vg[:, h // G])
            else:
                Kl, Vl = kv.get_local(l, m, p, s.window)
                for h in range(Hq):
                    y[h] = gated_attention_row(qr[h], Kg[:, h // G], Vg[:, h // G],
                                               Kl[:, h // G], Vl[:, h // G], z[h])  # Alg. 3 l.2-5
            x = x + np.asarray(W["wo"], np.float64) @ act_in(y.reshape(Hq * D), 1)      # Alg. 3 l.6
            b = act_in(rmsnorm(x, W["norm2"], s.norm_eps), 2)
            hid = (lambda t: act_in(t, 3)) if self.w_mx else None
            if s.n_experts > 0:
                x = x + moe_ffn(b, W, s.top_k, self.route_margins, hid)
            else:
                x = x + swiglu_ffn(b, W["w_gate"], W["w_up"], W["w_down"], hid)
            if self.layer_trace is not None:
                self.layer_trace.append((l, m, p, x_in.copy(), x.copy()))
        return x

    def embed(self, t):
        return np.asarray(self.w["emb"][int(t)], np.float64)

    def logits(self, h):
        return np.asarray(self._head, np.float64) @ rmsnorm(h, self.w["norm_f"], self.s.norm_eps)

    # -- Alg. 2: loop-serial over the whole sequence
    def seq_forward(self, tokens):
        """Returns H [L, n, d] (H[l-1, p] = loop-l state at position p) and logits [n, V]."""
        s = self.s
        n = len(tokens)
        kv = FullHistoryKV(self._store)
        E = np.stack([self.embed(t) for t in tokens])
        H = np.zeros((s.n_loops, n, s.d_model))
        for p in range(n):                                   # Alg. 2 l.2
            H[0, p] = self.f(E[p], p, 1, kv)
        for l in range(2, s.n_loops + 1):                    # Alg. 2 l.3-7
            shifted = np.concatenate([np.zeros((1, s.d_model)), H[l - 2, :-1]], axis=0)
            Bm = E + shifted
            for p in range(n):
                H[l - 1, p] = self.f(Bm[p], p, l, kv)
        lg = np.stack([self.logits(H[s.n_loops - 1, p]) for p in range(n)])   # Alg. 2 l.8
        return H, lg

    # -- Alg. 1: prefill, then one displaced micro-batch per new token
    def clp_prefill(self, tokens, max_ctx):
        """Alg. 1 l.1-3.  Consumes the prompt position by position with the same micro-batch
        rule as decoding (which equals Alg. 2 on the prompt); returns (next token id, logits)."""
        s = self.s
        self.kv = RingKV(self._store, s, max_ctx)
        self.carry = np.zeros((max(s.n_loops - 1, 0), s.d_model))   # carry[l-1] = H^l[p-1]
        self.pos = 0
        self.trace = []        # per position: H rows [L, d] (for tests)
        nxt, lg = None, None
        for t in tokens:
            nxt, lg = self.clp_decode_step(t)
        return nxt, lg

    def clp_decode_step(self, t):
        """Alg. 1 l.5-9 at position p = self.pos: rows B_0 = e, B_l = e + H^l[p-1]; one pass of f
        per row (rows are independent); carry update; head on the last loop's row."""
        s = self.s
        p = self.pos
        e = self.embed(t)
        rows = [e] + [e + self.carry[l - 1] for l in range(1, s.n_loops)]   # Alg. 1 l.6
        out = np.zeros((s.n_loops, s.d_model))
        # the first-loop row writes K_share/V_share[p] before the other rows read them:
        for l in range(1, s.n_loops + 1):
            out[l - 1] = self.f(rows[l - 1], p, l, self.kv)
        if s.n_loops > 1:
            self.carry = out[:-1].copy()
        lg = self.logits(out[-1])
        self.trace.append(out)
        self.pos = p + 1
        return int(np.argmax(lg)), lg

    # -- Eq. (1): vanilla loop transformer, every loop with its own full cache
    def vanilla_loop_forward(self, tokens):
        s = self.s
        n = len(tokens)
        kv = FullHistoryKV(self._store)
        H = np.zeros((s.n_loops, n, s.d_model))
        for p in range(n):
            h = self.embed(tokens[p])
            for l in range(1, s.n_loops + 1):
                h = self.f(h, p, l, kv, global_cache_id=l, plain=True)
                H[l - 1, p] = h
        lg = np.stack([self.logits(H[-1, p]) for p in range(n)])
        return H, lg

    def greedy_generate(self, prompt, n_new, max_ctx=None):
        """Alg. 1 end to end: returns n_new + 1 ids (the prefill's prediction and one per step),
        the top-2 logit margin of every prediction, and the logits of every prediction."""
        max_ctx = max_ctx or (len(prompt) + n_new + 1)
        nxt, lg = self.clp_prefill(prompt, max_ctx)
        ids, margins, all_lg = [nxt], [_margin(lg)], [lg]
        for _ in range(n_new):
            nxt, lg = self.clp_decode_step(nxt)
            ids.append(nxt); margins.append(_margin(lg)); all_lg.append(lg)
        return ids, margins, np.stack(all_lg)


def _margin(lg):
    top = np.sort(lg)[-2:]
    return float(top[1] - top[0])
