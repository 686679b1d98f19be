"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This module draws random numbers and rounds them to the storage type; it holds none of
the method's arithmetic (no attention, no norm, no RoPE, no GEMM).  Both sides receive
the very same values: the oracle as float64/float32 arrays, the HIP path as a packed
weight blob / device tensors made from those arrays.

All draws come from numpy's Philox counter-based generator keyed by (seed, stream id),
so a tensor's values depend only on its own stream id and shape, never on draw order.
"""
from __future__ import annotations

import dataclasses
import numpy as np


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Hyper-parameters of a PLT model (names follow the paper's notation where it has one)."""
    n_layers: int
    d_model: int
    n_heads: int       # H_q
    n_kv_heads: int    # H_kv
    head_dim: int      # D
    ffn_hidden: int    # F
    vocab: int         # V
    n_loops: int       # L
    window: int        # w
    rope_theta: float = 10000.0
    norm_eps: float = 1e-5
    tie_embeddings: bool = True
    n_experts: int = 0     # E; 0 = dense feed-forward, > 0: ffn_hidden is each expert's hidden size
    top_k: int = 0         # experts evaluated per row


TINY = ModelShape(n_layers=2, d_model=256, n_heads=4, n_kv_heads=4, head_dim=64,
                  ffn_hidden=1024, vocab=1024, n_loops=2, window=16)
PLT_1P3B = ModelShape(n_layers=24, d_model=2048, n_heads=16, n_kv_heads=16, head_dim=128,
                      ffn_hidden=5632, vocab=32000, n_loops=2, window=64)


# the paper's open-source dense recipe (appendix, "Dense Models Recipe"): 16 layers, hidden 2048, MLP hidden
# 16384, grouped-query attention with 32 query / 8 key-value heads, tied head (its extra norms are not modelled)
PLT_DENSE_GQA = ModelShape(n_layers=16, d_model=2048, n_heads=32, n_kv_heads=8, head_dim=64,
                           ffn_hidden=16384, vocab=50304, n_loops=2, window=64)


# the paper's open-source mixture-of-experts recipe (appendix, "MoE Models Recipe"): 16 layers, hidden 2048,
# 16 attention heads, SwiGLU experts, 8 of 64 per token; the expert hidden size is not printed -- 1024 (the
# value of the OLMoE model the recipe builds on) gives the quoted ~1B active / ~7B total parameters
PLT_MOE_1B7B = ModelShape(n_layers=16, d_model=2048, n_heads=16, n_kv_heads=16, head_dim=128,
                          ffn_hidden=1024, vocab=50304, n_loops=2, window=64, n_experts=64, top_k=8)
TINY_MOE = ModelShape(n_layers=2, d_model=256, n_heads=4, n_kv_heads=4, head_dim=64,
                      ffn_hidden=128, vocab=1024, n_loops=2, window=16, n_experts=8, top_k=2)


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, stream]))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of values that are already exactly representable in bfloat16."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def _e4m3_table() -> np.ndarray:
    """The 127 finite non-negative values of the 8-bit float e4m3 (OCP e4m3fn) by bit pattern
    0x00..0x7E: exponent field e (bias 7), mantissa m: 2^(e-7) (1 + m/8), subnormal m/8 * 2^-6."""
    code = np.arange(127)
    e, m = code >> 3, code & 7
    return np.where(e == 0, m / 8.0 * 2.0 ** -6, 2.0 ** (e - 7.0) * (1 + m / 8.0)).astype(np.float32)


def e4m3_bits(x: np.ndarray) -> np.ndarray:
    """uint8 e4m3 codes nearest to x (ties to the even code, saturating at +-448)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    tab = _e4m3_table().astype(np.float64)
    mag = np.minimum(np.abs(x.astype(np.float64)), 448.0)
    hi = np.clip(np.searchsorted(tab, mag, side="left"), 1, 126)       # tab[hi-1] <= mag <= tab[hi]
    lo = hi - 1
    dl, dh = mag - tab[lo], tab[hi] - mag
    code = np.where(dl < dh, lo, np.where(dh < dl, hi, np.where(lo % 2 == 0, lo, hi)))
    return (code | np.where(np.signbit(x), 0x80, 0)).astype(np.uint8).reshape(x.shape)


def e4m3_from_bits(b: np.ndarray) -> np.ndarray:
    b = np.asarray(b, np.uint8)
    v = _e4m3_table()[np.minimum(b & 0x7F, 126)]
    return np.where(b & 0x80, -v, v).astype(np.float32).reshape(b.shape)


def e2m1_from_bits(b: np.ndarray) -> np.ndarray:
    """Values of 4-bit e2m1 codes (bit 3 sign; magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6 by code 0..7)."""
    b = np.asarray(b, np.uint8)
    v = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], np.float32)[b & 7]
    return np.where(b & 8, -v, v).astype(np.float32)


def round_to_e4m3(x: np.ndarray) -> np.ndarray:
    return e4m3_from_bits(e4m3_bits(x))


def normal(shape, seed: int, stream: int, std: float = 1.0, bf16: bool = False) -> np.ndarray:
    x = _rng(seed, stream).standard_normal(size=shape, dtype=np.float32) * np.float32(std)
    return round_to_bf16(x) if bf16 else x


def token_ids(shape, vocab: int, seed: int, stream: int = 1000) -> np.ndarray:
    return _rng(seed, stream).integers(0, vocab, size=shape, dtype=np.int64).astype(np.int32)


def make_weights(shape: ModelShape, seed: int, bf16: bool, std: float = 0.02,
                 gate_std: float | None = None, router_std: float | None = None) -> dict:
    """Weights N(0, std); norm gains 1; gate bias 0.  Matrices are [out_features, in_features].

    Returns {"emb", "norm_f", "head" (absent when tied), "layers": [ {...} ]}, float32 arrays
    whose values are bf16-representable when bf16=True.  Mixture-of-experts shapes: "router" [E, d] and
    "w_gate" / "w_up" [E, F, d], "w_down" [E, d, F].
    """
    s = shape
    hq, hkv, dh, d, f = s.n_heads, s.n_kv_heads, s.head_dim, s.d_model, s.ffn_hidden
    gstd = std if gate_std is None else gate_std
    rstd = std if router_std is None else router_std
    E = shape.n_experts
    ex = (E,) if E > 0 else ()       # expert matrices carry a leading expert axis
    w = {"emb": normal((s.vocab, d), seed, 1, std, bf16),
         "norm_f": np.ones(d, np.float32), "layers": []}
    if not s.tie_embeddings:
        w["head"] = normal((s.vocab, d), seed, 2, std, bf16)
    for m in range(s.n_layers):
        base = 100 + 16 * m
        layer = {
            "norm1": np.ones(d, np.float32),
            "wq": normal((hq * dh, d), seed, base + 0, std, bf16),
            "wk": normal((hkv * dh, d), seed, base + 1, std, bf16),
            "wv": normal((hkv * dh, d), seed, base + 2, std, bf16),
            "gate_w": normal((hq, dh), seed, base + 3, gstd, bf16),
            "gate_b": np.zeros(hq, np.float32),
            "wo": normal((d, hq * dh), seed, base + 4, std, bf16),
            "norm2": np.ones(d, np.float32),
            "w_gate": normal(ex + (f, d), seed, base + 5, std, bf16),
            "w_up": normal(ex + (f, d), seed, base + 6, std, bf16),
            "w_down": normal(ex + (d, f), seed, base + 7, std, bf16),
        }
        if E > 0:
            layer["router"] = normal((E, d), seed, base + 8, rstd, bf16)
        w["layers"].append(layer)
    return w


def make_attn_inputs(B: int, L: int, Hq: int, Hkv: int, D: int, N: int, w: int,
                     seed: int, bf16: bool) -> dict:
    """Inputs of the kernel-only fused decode attention: all N(0,1).

    q [B,L,Hq,D]; k_share, v_share [B,Hkv,N,D]; k_ring, v_ring [B,L-1,Hkv,w,D] (slot order);
    z [B,L-1,Hq] gate logits (float32, never rounded).
    """
    out = {
        "q": normal((B, L, Hq, D), seed, 10, 1.0, bf16),
        "k_share": normal((B, Hkv, N, D), seed, 11, 1.0, bf16),
        "v_share": normal((B, Hkv, N, D), seed, 12, 1.0, bf16),
        "k_ring": normal((B, max(L - 1, 0), Hkv, w, D), seed, 13, 1.0, bf16),
        "v_ring": normal((B, max(L - 1, 0), Hkv, w, D), seed, 14, 1.0, bf16),
        "z": normal((B, max(L - 1, 0), Hq), seed, 15, 1.0, False),
    }
    return out
