"""Independent float64 torch routines the oracle is pinned against (CPU only).

None of this is used by the oracle or by the HIP path.  It is a second formulation,
token-parallel and mask-based, built from library routines: torch's
scaled_dot_product_attention, rms_norm and silu, and RoPE in the complex-number form
x_j + i x_{j+D/2} -> (x_j + i x_{j+D/2}) * exp(i p theta^(-2j/D)).
"""
import torch
import torch.nn.functional as F


def t64(a):
    return torch.as_tensor(a, dtype=torch.float64)


def rope_complex(x, theta):
    """x [n, H, D] at positions 0..n-1."""
    n, H, D = x.shape
    half = D // 2
    zc = torch.complex(x[..., :half], x[..., half:])
    pos = torch.arange(n, dtype=torch.float64)[:, None]
    freq = theta ** (-torch.arange(half, dtype=torch.float64) * 2.0 / D)[None, :]
    rot = torch.polar(torch.ones(n, half, dtype=torch.float64), pos * freq)[:, None, :]
    out = zc * rot
    return torch.cat([out.real, out.imag], dim=-1)


def _expand_kv(k, G):
    return k.repeat_interleave(G, dim=1)


def decoder_stack(X, weights, shape, shared_kv=None, window=None, return_kv=False):
    """Textbook pre-norm decoder stack on a whole sequence X [n, d].

    shared_kv=None: plain causal self-attention (a standard transformer).
    shared_kv=[(K_m, V_m)] per layer: PLT non-first loop -- causal attention over the given
    keys/values plus banded (window) causal attention over this pass's own K/V, merged by
    the per-head sigmoid gate on the un-rotated queries.
    """
    s = shape
    n = X.shape[0]
    Hq, Hkv, D = s.n_heads, s.n_kv_heads, s.head_dim
    G = Hq // Hkv
    idx = torch.arange(n)
    causal = idx[None, :] <= idx[:, None]
    kv_out = []
    x = X.clone()
    for m in range(s.n_layers):
        W = weights["layers"][m]
        a = F.rms_norm(x, (s.d_model,), t64(W["norm1"]), s.norm_eps)
        q = F.linear(a, t64(W["wq"])).view(n, Hq, D)
        k = F.linear(a, t64(W["wk"])).view(n, Hkv, D)
        v = F.linear(a, t64(W["wv"])).view(n, Hkv, D)
        qr, kr = rope_complex(q, s.rope_theta), rope_complex(k, s.rope_theta)
        kv_out.append((kr, v))
        qh = qr.transpose(0, 1)                                   # [Hq, n, D]
        own = F.scaled_dot_product_attention(
            qh, _expand_kv(kr, G).transpose(0, 1), _expand_kv(v, G).transpose(0, 1),
            attn_mask=(causal if window is None else causal & (idx[None, :] > idx[:, None] - window)))
        if shared_kv is None:
            y = own
        else:
            Ks, Vs = shared_kv[m]
            glob = F.scaled_dot_product_attention(
                qh, _expand_kv(Ks, G).transpose(0, 1), _expand_kv(Vs, G).transpose(0, 1), attn_mask=causal)
            z = torch.einsum("nhd,hd->nh", q, t64(W["gate_w"])) + t64(W["gate_b"])
            g = torch.sigmoid(z).transpose(0, 1)[..., None]          # [Hq, n, 1]
            y = g * own + (1 - g) * glob
        x = x + F.linear(y.transpose(0, 1).reshape(n, Hq * D), t64(W["wo"]))
        b = F.rms_norm(x, (s.d_model,), t64(W["norm2"]), s.norm_eps)
        if getattr(s, "n_experts", 0) > 0:
            x = x + moe_ffn_dense(b, W, s.top_k)
        else:
            x = x + F.linear(F.silu(F.linear(b, t64(W["w_gate"]))) * F.linear(b, t64(W["w_up"])), t64(W["w_down"]))
    return (x, kv_out) if return_kv else x


def moe_ffn_dense(b, W, top_k):
    """Mixture-of-experts feed-forward, token-parallel and dense: every expert is evaluated on every
    row b [n, d] (batched matmuls), and a 0/1 mask built from torch.topk of the softmax probabilities
    keeps the top_k experts of each row, weighted by their probabilities as they are."""
    prob = torch.softmax(F.linear(b, t64(W["router"])), dim=-1)                    # [n, E]
    keep = torch.zeros_like(prob).scatter_(1, torch.topk(prob, top_k, dim=-1).indices, 1.0)
    gate = torch.einsum("efd,nd->nef", t64(W["w_gate"]), b)
    up = torch.einsum("efd,nd->nef", t64(W["w_up"]), b)
    out = torch.einsum("edf,nef->ned", t64(W["w_down"]), F.silu(gate) * up)        # [n, E, d]
    return torch.einsum("ne,ned->nd", prob * keep, out)


def head_logits(H, weights, shape):
    hw = weights["emb"] if shape.tie_embeddings else weights["head"]
    return F.linear(F.rms_norm(H, (shape.d_model,), t64(weights["norm_f"]), shape.norm_eps), t64(hw))


def plt_forward(tokens, weights, shape, variant="plt"):
    """Token-parallel, loop-serial PLT forward (training-time form): returns H [L, n, d], logits.
    variant "clp_own_kv": every loop is a plain stack on E + shift(H) (own KV, no sharing, no gate)."""
    E = t64(weights["emb"])[torch.as_tensor(tokens, dtype=torch.long)]
    H1, kv = decoder_stack(E, weights, shape, return_kv=True)
    Hs = [H1]
    for _ in range(1, shape.n_loops):
        shifted = torch.cat([torch.zeros(1, shape.d_model, dtype=torch.float64), Hs[-1][:-1]], dim=0)
        if variant == "clp_own_kv":
            Hs.append(decoder_stack(E + shifted, weights, shape))
        else:
            Hs.append(decoder_stack(E + shifted, weights, shape, shared_kv=kv, window=shape.window))
    return torch.stack(Hs), head_logits(Hs[-1], weights, shape)


def vanilla_loop_forward(tokens, weights, shape):
    E = t64(weights["emb"])[torch.as_tensor(tokens, dtype=torch.long)]
    Hs, h = [], E
    for _ in range(shape.n_loops):
        h = decoder_stack(h, weights, shape)
        Hs.append(h)
    return torch.stack(Hs), head_logits(h, weights, shape)
