"""Shared helpers of the GPU parity tests (inputs, oracle shape conversion)."""
import numpy as np

from oracle import plt_oracle as O
from paper_2510_24824_amd import synth


def oshape(s, **kw):
    d = dict(n_layers=s.n_layers, d_model=s.d_model, n_heads=s.n_heads, n_kv_heads=s.n_kv_heads,
             head_dim=s.head_dim, ffn_hidden=s.ffn_hidden, vocab=s.vocab, n_loops=s.n_loops,
             window=s.window, rope_theta=s.rope_theta, norm_eps=s.norm_eps, tie_embeddings=s.tie_embeddings,
             n_experts=s.n_experts, top_k=s.top_k)
    d.update(kw)
    return O.OracleShape(**d)


def with_shape(s, **kw):
    return synth.ModelShape(**{**s.__dict__, **kw})


def lively_weights(shape, seed, bf16, std=0.02, gate_std=0.5, router_std=None):
    """Paper-style N(0, std) weights, but with non-trivial norm gains, gate weights and gate
    biases so that every parameter tensor influences the result."""
    w = synth.make_weights(shape, seed, bf16=bf16, std=std, gate_std=gate_std, router_std=router_std)
    rng = np.random.default_rng(seed + 17)
    for lw in w["layers"]:
        lw["gate_b"] = (0.5 * rng.standard_normal(shape.n_heads)).astype(np.float32)
        lw["norm1"] = (1 + 0.1 * rng.standard_normal(shape.d_model)).astype(np.float32)
        lw["norm2"] = (1 + 0.1 * rng.standard_normal(shape.d_model)).astype(np.float32)
    w["norm_f"] = (1 + 0.1 * rng.standard_normal(shape.d_model)).astype(np.float32)
    return w
