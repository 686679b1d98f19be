"""Pins of the oracle's mixture-of-experts feed-forward (CPU only): library routines, closed forms and
an independent dense, token-parallel formulation -- and planted mistakes that the pins must catch."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import plt_oracle as O
from paper_2510_24824_amd import synth
from tests import textbook as T
from tests.test_oracle_pins import oshape

SMALL_MOE = synth.ModelShape(n_layers=2, d_model=32, n_heads=4, n_kv_heads=2, head_dim=8, ffn_hidden=24,
                             vocab=37, n_loops=3, window=4, n_experts=6, top_k=2)


def moe_weights(shape=SMALL_MOE, seed=3, std=0.3):
    w = synth.make_weights(shape, seed, bf16=False, std=std, gate_std=1.0, router_std=0.5)
    rng = np.random.default_rng(seed)
    for lw in w["layers"]:
        lw["gate_b"] = rng.standard_normal(shape.n_heads).astype(np.float32)
        lw["norm2"] = (1 + 0.1 * rng.standard_normal(shape.d_model)).astype(np.float32)
    return w


def _layer(seed=4, E=6, F_=24, d=32):
    sh = synth.ModelShape(**{**SMALL_MOE.__dict__, "n_experts": E, "ffn_hidden": F_, "d_model": d, "n_layers": 1})
    return moe_weights(sh, seed)["layers"][0]


def test_route_matches_library_softmax_and_topk():
    rng = np.random.default_rng(0)
    W = _layer()
    for _ in range(20):
        b = rng.standard_normal(32)
        ids, p, margin = O.moe_route(b, W["router"], 3)
        prob = torch.softmax(T.t64(W["router"]) @ T.t64(b), dim=0)
        top = torch.topk(prob, 3)
        assert list(ids) == top.indices.tolist()                       # decreasing probability
        assert np.max(np.abs(p - top.values.numpy())) < 1e-14
        lg = np.sort(np.asarray(W["router"], np.float64) @ b)[::-1]
        assert abs(margin - (lg[2] - lg[3])) < 1e-12
    assert O.moe_route(b, W["router"], 6)[2] == math.inf


def test_moe_ffn_equals_dense_masked_formulation():
    rng = np.random.default_rng(1)
    W = _layer()
    B = rng.standard_normal((9, 32))
    want = T.moe_ffn_dense(T.t64(B), W, 2).numpy()
    got = np.stack([O.moe_ffn(b, W, 2) for b in B])
    assert np.max(np.abs(got - want)) < 1e-12


def test_single_expert_is_the_dense_ffn():
    W = _layer(E=1)
    b = np.random.default_rng(2).standard_normal(32)
    want = F.linear(F.silu(F.linear(T.t64(b), T.t64(W["w_gate"][0]))) * F.linear(T.t64(b), T.t64(W["w_up"][0])),
                    T.t64(W["w_down"][0])).numpy()
    assert np.max(np.abs(O.moe_ffn(b, W, 1) - want)) < 1e-12        # softmax over one expert is 1
    assert np.max(np.abs(O.swiglu_ffn(b, W["w_gate"][0], W["w_up"][0], W["w_down"][0]) - want)) < 1e-12


def test_identical_experts_scale_by_the_selected_probability_mass():
    """With equal experts the output is (sum of the selected p) * FFN(b): 1 for top_k = E, and for
    top_k < E the un-renormalised mass, here from router logits fixed by construction."""
    W = _layer(E=4)
    for name in ("w_gate", "w_up", "w_down"):
        W[name] = np.repeat(W[name][:1], 4, axis=0)
    b = np.zeros(32); b[0] = 1.0
    W["router"] = np.zeros((4, 32), np.float32); W["router"][:, 0] = np.log([1.0, 2.0, 3.0, 4.0])   # p = [.1 .2 .3 .4]
    one = O.swiglu_ffn(b, W["w_gate"][0], W["w_up"][0], W["w_down"][0])
    assert np.max(np.abs(O.moe_ffn(b, W, 4) - one)) < 1e-12
    assert np.max(np.abs(O.moe_ffn(b, W, 2) - 0.7 * one)) < 1e-7
    assert np.max(np.abs(O.moe_ffn(b, W, 1) - 0.4 * one)) < 1e-7
    ids, p, _ = O.moe_route(b, W["router"], 3)
    assert list(ids) == [3, 2, 1] and np.max(np.abs(p - [0.4, 0.3, 0.2])) < 1e-7


def test_distinct_experts_get_their_own_probability():
    """Two experts, both selected: out = p0 FFN_0 + p1 FFN_1 with p from the two-way closed form."""
    W = _layer(E=2)
    b = np.random.default_rng(5).standard_normal(32)
    r = np.asarray(W["router"], np.float64) @ b
    p0 = 1.0 / (1.0 + math.exp(r[1] - r[0]))
    f0 = O.swiglu_ffn(b, W["w_gate"][0], W["w_up"][0], W["w_down"][0])
    f1 = O.swiglu_ffn(b, W["w_gate"][1], W["w_up"][1], W["w_down"][1])
    assert np.max(np.abs(O.moe_ffn(b, W, 2) - (p0 * f0 + (1 - p0) * f1))) < 1e-12


def test_equal_probabilities_take_the_lowest_indices():
    W = _layer(E=5)
    W["router"] = np.zeros_like(W["router"])
    ids, p, margin = O.moe_route(np.ones(32), W["router"], 2)
    assert list(ids) == [0, 1] and np.allclose(p, 0.2) and margin == 0.0


@pytest.mark.parametrize("L,k", [(1, 2), (3, 2), (2, 6)])
def test_moe_model_equals_token_parallel_formulation_and_clp(L, k):
    """Whole model: Alg. 2 with the MoE feed-forward against the mask-based torch stack, and
    cross-loop-parallel decoding (Alg. 1) against Alg. 2."""
    ms = synth.ModelShape(**{**SMALL_MOE.__dict__, "n_loops": L, "top_k": k})
    shape, wts = oshape(ms, n_experts=ms.n_experts, top_k=k), moe_weights(ms)
    toks = synth.token_ids((10,), ms.vocab, seed=7)
    orc = O.PLTOracle(shape, wts)
    H, lg = orc.seq_forward(toks)
    Ht, lgt = T.plt_forward(toks, wts, shape)
    assert np.max(np.abs(H - Ht.numpy())) < 1e-10 and np.max(np.abs(lg - lgt.numpy())) < 1e-10
    assert len(orc.route_margins) == L * 10 * ms.n_layers
    orc.clp_prefill(toks[:4], max_ctx=16)
    for t in toks[4:]:
        orc.clp_decode_step(t)
    assert np.max(np.abs(np.stack(orc.trace).transpose(1, 0, 2) - H)) < 1e-10


# ---- planted mistakes
PINS = [test_route_matches_library_softmax_and_topk, test_moe_ffn_equals_dense_masked_formulation,
        test_single_expert_is_the_dense_ffn, test_identical_experts_scale_by_the_selected_probability_mass,
        test_distinct_experts_get_their_own_probability, test_equal_probabilities_take_the_lowest_indices,
        lambda: test_moe_model_equals_token_parallel_formulation_and_clp(3, 2)]


def some_pin_fails():
    for pin in PINS:
        try:
            pin()
        except AssertionError:
            return True
    return False


def _route_variant(kind):
    def route(b, router, top_k):
        r = np.asarray(router, np.float64) @ np.asarray(b, np.float64)
        e = np.exp(r - np.max(r)); p = e / np.sum(e)
        order = np.argsort(-p, kind="stable")
        if kind == "smallest":
            order = np.argsort(p, kind="stable")
        if kind == "ties_high":
            order = np.argsort(-p[::-1], kind="stable"); order = len(p) - 1 - order
        ids = order[:top_k - 1] if kind == "one_short" and top_k > 1 else order[:top_k]
        w = p[ids]
        if kind == "renormalised":
            w = w / np.sum(w)
        if kind == "logit_weights":
            w = r[ids]
        if kind == "weights_reversed":
            w = w[::-1]
        if kind == "no_softmax_shift":          # softmax of r without the other experts: sigmoid-like weights
            w = 1.0 / (1.0 + np.exp(-r[ids]))
        margin = float(r[order[top_k - 1]] - r[order[top_k]]) if top_k < len(r) else math.inf
        return ids, w, margin
    return route


@pytest.mark.parametrize("kind", ["smallest", "ties_high", "one_short", "renormalised", "logit_weights",
                                  "weights_reversed", "no_softmax_shift"])
def test_route_mutations_are_caught(monkeypatch, kind):
    assert not some_pin_fails()
    monkeypatch.setattr(O, "moe_route", _route_variant(kind))
    assert some_pin_fails()


def _ffn_no_up(b, w_gate, w_up, w_down, hidden_in=None):
    g = np.asarray(w_gate, np.float64) @ b
    return np.asarray(w_down, np.float64) @ (g / (1.0 + np.exp(-g)))


def _ffn_silu_on_up(b, w_gate, w_up, w_down, hidden_in=None):
    g = np.asarray(w_gate, np.float64) @ b; u = np.asarray(w_up, np.float64) @ b
    return np.asarray(w_down, np.float64) @ (g * (u / (1.0 + np.exp(-u))))


@pytest.mark.parametrize("repl", [_ffn_no_up, _ffn_silu_on_up])
def test_expert_ffn_mutations_are_caught(monkeypatch, repl):
    monkeypatch.setattr(O, "swiglu_ffn", repl)
    assert some_pin_fails()


def test_wrong_expert_matrix_is_caught(monkeypatch):
    def moe_ffn(b, W, top_k, margins=None, hidden_in=None):
        ids, p, margin = O.moe_route(b, W["router"], top_k)
        out = np.zeros(np.asarray(W["w_down"]).shape[1])
        for e, pe in zip(ids, p):
            out += pe * O.swiglu_ffn(b, W["w_gate"][e], W["w_up"][e], W["w_down"][ids[0]])   # first expert's down matrix
        if margins is not None:
            margins.append(margin)
        return out
    monkeypatch.setattr(O, "moe_ffn", moe_ffn)
    assert some_pin_fails()
