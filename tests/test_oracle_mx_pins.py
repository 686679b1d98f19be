"""Pins of the oracle's microscaling quantisation (CPU only): the formats' value tables, brute-force nearest
search, closed forms, torch's own e4m3 conversion, hand-worked blocks -- and planted mistakes."""
import itertools
import math

import numpy as np
import pytest
import torch

from oracle import plt_oracle as O
from paper_2510_24824_amd import synth
from tests.test_oracle_pins import SMALL, oshape, small_weights

E2M1 = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])     # by code 0..7: exponent field e, mantissa m (bias 1)


def test_e2m1_table_follows_the_format_definition():
    for code in range(8):
        e, m = code >> 1, code & 1
        want = m / 2.0 if e == 0 else 2.0 ** (e - 1) * (1 + m / 2.0)
        assert E2M1[code] == want
    assert np.array_equal(O.e2m1_round(E2M1), E2M1) and np.array_equal(O.e2m1_round(-E2M1), -E2M1)


def _nearest_even_code(v):
    d = np.abs(E2M1 - min(abs(v), 6.0))
    best = np.flatnonzero(d == d.min())
    code = best[0] if len(best) == 1 else [c for c in best if c % 2 == 0][0]      # tie: even mantissa bit
    return math.copysign(E2M1[code], v)


def test_e2m1_round_is_the_nearest_value_ties_to_even_saturating():
    rng = np.random.default_rng(0)
    xs = np.concatenate([rng.uniform(-8, 8, 4000), rng.normal(0, 1, 2000),
                         [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, -0.25, -2.5, -5.0, 6.9, 7.0, 100.0, -1e9, 1e-9]])
    got = O.e2m1_round(xs)
    want = np.array([_nearest_even_code(v) for v in xs])
    assert np.array_equal(got, want)
    # the ties, spelled out: 0.25 -> 0, 0.75 -> 1, 1.25 -> 1, 1.75 -> 2, 2.5 -> 2, 3.5 -> 4, 5 -> 4
    assert list(O.e2m1_round(np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]))) == [0.0, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0]


def test_mx_scale_is_the_power_of_two_that_puts_the_block_maximum_in_the_top_binade():
    rng = np.random.default_rng(1)
    x = rng.normal(0, 1, (50, 64)) * np.exp(rng.uniform(-20, 20, (50, 1)))
    for fmt, emax, top in (("e2m1", 2, 6.0), ("e4m3", 8, 448.0)):
        q, e = O.mx_quantize(x, fmt)
        assert e.shape == (50, 2) and e.dtype.kind == "i"
        amax = np.abs(x.reshape(50, 2, 32)).max(-1)
        scaled = amax / 2.0 ** e
        assert np.all(scaled >= 2.0 ** emax) and np.all(scaled < 2.0 ** (emax + 1))
        assert np.all(e == np.floor(np.log2(amax)).astype(int) - emax)
        assert np.max(np.abs(q)) <= top
    # hand-worked block: maximum 5.0 -> floor(log2 5) = 2 -> e = 0 for e2m1; elements rounded on the grid
    blk = np.zeros(32); blk[:6] = [5.0, -2.4, 0.26, 0.74, 3.6, -7.9e-1]
    q, e = O.mx_quantize(blk, "e2m1")
    assert e[0] == 0 and list(q[:6]) == [4.0, -2.0, 0.5, 0.5, 4.0, -1.0]
    # maximum 0.3 -> floor(log2) = -2 -> e = -4: 0.3 * 16 = 4.8 -> 4 (tie rule not involved), 0.1 * 16 = 1.6 -> 1.5
    blk = np.zeros(32); blk[:2] = [0.3, 0.1]
    q, e = O.mx_quantize(blk, "e2m1")
    assert e[0] == -4 and list(q[:2]) == [4.0, 1.5]
    assert np.allclose(O.mx_dequantize(q, e)[:2], [0.25, 0.09375])
    # e4m3 block with maximum 1.0: e = -8, 1.0 -> 256
    blk = np.zeros(32); blk[:3] = [1.0, -0.5, 0.3]
    q, e = O.mx_quantize(blk, "e4m3")
    assert e[0] == -8 and list(q[:3]) == [256.0, -128.0, 80.0]        # 0.3 * 256 = 76.8 -> grid step 8 in [64, 128)


def test_mx_zero_block_and_exact_round_trip():
    q, e = O.mx_quantize(np.zeros(64), "e2m1")
    assert np.all(q == 0) and np.all(e == -127)
    rng = np.random.default_rng(2)
    # values that are grid points times a common power of two survive exactly (when the block holds a top-binade value)
    for fmt, grid in (("e2m1", E2M1), ("e4m3", synth.e4m3_from_bits(np.arange(127, dtype=np.uint8)).astype(np.float64))):
        top = grid[-1]
        for _ in range(20):
            vals = rng.choice(grid, 32) * rng.choice([-1.0, 1.0], 32)
            vals[0] = top
            sh = int(rng.integers(-30, 30))
            q, e = O.mx_quantize(vals * 2.0 ** sh, fmt)
            assert np.array_equal(O.mx_dequantize(q, e), vals * 2.0 ** sh)


def test_mx_e4m3_elements_match_torch_conversion():
    rng = np.random.default_rng(3)
    x = rng.normal(0, 1, (8, 96)).astype(np.float32).astype(np.float64)
    q, e = O.mx_quantize(x, "e4m3")
    scaled = (x.reshape(8, 3, 32) * 2.0 ** (-e)[..., None]).reshape(8, 96)
    # torch's cast does not saturate (it yields NaN beyond the largest value); the block scale leaves scaled
    # magnitudes up to 512, and those above 448 must come out as 448
    inside = np.abs(scaled) <= 448.0
    want = torch.tensor(np.where(inside, scaled, 0.0), dtype=torch.float32).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(q[inside], want[inside])
    assert (~inside).sum() >= 2 and np.array_equal(q[~inside], np.sign(scaled[~inside]) * 448.0)


def test_mx_error_bounds():
    rng = np.random.default_rng(4)
    x = rng.normal(0, 1, (200, 32))
    for fmt, emax, mant in (("e2m1", 2, 1), ("e4m3", 8, 3)):
        q, e = O.mx_quantize(x, fmt)
        err = np.abs(O.mx_dequantize(q, e) - x)
        amax = np.abs(x).max(-1, keepdims=True)
        # half a grid step of the top binade, or the saturation gap between 2^(emax+1) and the largest value
        sat = 2.0 ** (emax + 1) - (6.0 if fmt == "e2m1" else 448.0)
        assert np.all(err <= 2.0 ** e * max(2.0 ** (emax - mant - 1), sat) + 1e-300)
        assert np.all(err <= amax * 0.26)


def test_mx_linear_equals_explicit_block_sums():
    """y_n = sum over blocks 2^(ea_b + ew_nb) * sum_k qa_k qw_nk, with integer-valued inner sums."""
    rng = np.random.default_rng(5)
    a = rng.normal(0, 1, 96); W = rng.normal(0, 0.05, (7, 96))
    wq, we = O.mx_quantize(W, "e2m1")
    aq, ae = O.mx_quantize(a, "e4m3")
    want = np.zeros(7)
    for n, b in itertools.product(range(7), range(3)):
        inner = float(np.sum(aq[32 * b:32 * b + 32] * wq[n, 32 * b:32 * b + 32]))
        assert inner * 16 == round(inner * 16)                       # products of grid values: multiples of 1/16
        want[n] += 2.0 ** (int(ae[b]) + int(we[n, b])) * inner
    assert np.max(np.abs(O.mx_linear(a, wq, we) - want)) <= 1e-12 * np.max(np.abs(want))
    # and the quantised product stays close to the exact one
    assert np.max(np.abs(O.mx_linear(a, wq, we) - W @ a)) <= 0.2 * np.linalg.norm(W, axis=1).max() * np.linalg.norm(a) / math.sqrt(96) * 3


def test_model_with_mx_linear_layers_equals_a_model_on_dequantised_weights_and_quantised_inputs():
    """w_mx=True is the ordinary oracle run on dequantised weights, with the projection inputs passed through
    the e4m3 block quantiser: checked by replaying one layer by hand from the oracle's own building blocks
    with independent quantiser calls."""
    ms = synth.ModelShape(**{**SMALL.__dict__, "ffn_hidden": 64, "n_loops": 1, "n_layers": 1})   # every K a multiple of 32
    shape = oshape(ms)
    wts = small_weights(shape=ms)
    toks = synth.token_ids((5,), SMALL.vocab, seed=3)
    H, lg = O.PLTOracle(shape, wts, w_mx=True).seq_forward(toks)
    # position 0 by hand (one key: attention returns v)
    W = wts["layers"][0]
    dq = lambda M: O.mx_dequantize(*O.mx_quantize(M, "e2m1"))
    qa = lambda t: O.mx_dequantize(*O.mx_quantize(t, "e4m3"))
    x = wts["emb"][toks[0]].astype(np.float64)
    a = qa(O.rmsnorm(x, W["norm1"], shape.norm_eps))
    v = (dq(W["wv"]) @ a).reshape(shape.n_kv_heads, shape.head_dim)
    y = np.repeat(v, shape.n_heads // shape.n_kv_heads, axis=0).reshape(-1)
    x = x + dq(W["wo"]) @ qa(y)
    b = qa(O.rmsnorm(x, W["norm2"], shape.norm_eps))
    g = dq(W["w_gate"]) @ b
    x = x + dq(W["w_down"]) @ qa(g / (1 + np.exp(-g)) * (dq(W["w_up"]) @ b))
    assert np.max(np.abs(H[0, 0] - x)) < 1e-10
    # and it differs from the unquantised model by a quantisation-sized amount, not by zero
    H0, _ = O.PLTOracle(shape, wts).seq_forward(toks)
    rel = np.max(np.abs(H - H0)) / np.max(np.abs(H0))
    assert 1e-3 < rel < 1.5


def test_moe_model_with_mx_experts_equals_hand_composition():
    """Mixture-of-experts feed-forward on low-bit operands, one position by hand: the router reads the quantised
    normed row with its own (unquantised) matrix; every selected expert runs on dequantised e2m1 matrices, its
    hidden vector passes the e4m3 quantiser before the down projection."""
    ms = synth.ModelShape(n_layers=1, d_model=32, n_heads=4, n_kv_heads=2, head_dim=8, ffn_hidden=32, vocab=37,
                          n_loops=1, window=4, n_experts=5, top_k=2)
    shape = oshape(ms, n_experts=5, top_k=2)
    wts = synth.make_weights(ms, 4, bf16=False, std=0.3, gate_std=1.0, router_std=0.5)
    toks = synth.token_ids((3,), ms.vocab, seed=5)
    H, _ = O.PLTOracle(shape, wts, w_mx=True).seq_forward(toks)
    W = wts["layers"][0]
    dq = lambda M: O.mx_dequantize(*O.mx_quantize(M, "e2m1"))
    qa = lambda t: O.mx_dequantize(*O.mx_quantize(t, "e4m3"))
    x = wts["emb"][toks[0]].astype(np.float64)
    a = qa(O.rmsnorm(x, W["norm1"], shape.norm_eps))
    v = (dq(W["wv"]) @ a).reshape(shape.n_kv_heads, shape.head_dim)
    x = x + dq(W["wo"]) @ qa(np.repeat(v, 2, axis=0).reshape(-1))
    b = qa(O.rmsnorm(x, W["norm2"], shape.norm_eps))
    r = W["router"].astype(np.float64) @ b
    p = np.exp(r - r.max()); p /= p.sum()
    top = np.argsort(-p)[:2]
    for e in top:
        g = dq(W["w_gate"][e]) @ b
        x = x + p[e] * (dq(W["w_down"][e]) @ qa(g / (1 + np.exp(-g)) * (dq(W["w_up"][e]) @ b)))
    assert np.max(np.abs(H[0, 0] - x)) < 1e-10


# ---- planted mistakes
PINS = [test_e2m1_round_is_the_nearest_value_ties_to_even_saturating,
        test_mx_scale_is_the_power_of_two_that_puts_the_block_maximum_in_the_top_binade,
        test_mx_zero_block_and_exact_round_trip, test_mx_e4m3_elements_match_torch_conversion,
        test_mx_error_bounds, test_mx_linear_equals_explicit_block_sums,
        test_model_with_mx_linear_layers_equals_a_model_on_dequantised_weights_and_quantised_inputs,
        test_moe_model_with_mx_experts_equals_hand_composition]


def some_pin_fails():
    for pin in PINS:
        try:
            pin()
        except AssertionError:
            return True
    return False


def _e2m1_ties_away(x):
    a = np.clip(np.asarray(x, np.float64), -6.0, 6.0); mag = np.abs(a)
    _, ex = np.frexp(mag); step = np.ldexp(1.0, np.maximum(ex - 1, 0) - 1)
    return np.sign(a) * np.minimum(np.floor(mag / step + 0.5) * step, 6.0)


def _e2m1_no_subnormal(x):
    a = np.clip(np.asarray(x, np.float64), -6.0, 6.0); mag = np.abs(a)
    _, ex = np.frexp(mag); step = np.ldexp(1.0, np.maximum(ex - 1, 0) - 1)
    r = np.minimum(np.rint(mag / step) * step, 6.0)
    return np.sign(a) * np.where(r == 0.5, 0.0, r)


def _e2m1_no_saturation(x):
    a = np.asarray(x, np.float64); mag = np.abs(a)
    _, ex = np.frexp(mag); step = np.ldexp(1.0, np.maximum(ex - 1, 0) - 1)
    return np.sign(a) * np.rint(mag / step) * step


@pytest.mark.parametrize("repl", [_e2m1_ties_away, _e2m1_no_subnormal, _e2m1_no_saturation])
def test_e2m1_mutations_are_caught(monkeypatch, repl):
    assert not some_pin_fails()
    monkeypatch.setattr(O, "e2m1_round", repl)
    monkeypatch.setitem(O._MX_FORMATS, "e2m1", (2, repl))
    assert some_pin_fails()


def _mx_variant(kind):
    def mx_quantize(x, fmt):
        emax, rnd = O._MX_FORMATS[fmt]
        x = np.asarray(x, np.float64); K = x.shape[-1]
        blk = x.reshape(*x.shape[:-1], K // 32, 32)
        if kind == "block_16":
            blk = x.reshape(*x.shape[:-1], K // 16, 16)
        amax = np.max(np.abs(blk), axis=-1)
        _, ex = np.frexp(amax)
        fl = ex - 1
        if kind == "ceil_log2":
            fl = np.ceil(np.log2(np.where(amax > 0, amax, 1.0))).astype(int)
        em = emax + 1 if kind == "emax_plus_one" else emax - 1 if kind == "emax_minus_one" else emax
        e = np.where(amax > 0, np.clip(fl - em, -127, 127), -127).astype(np.int64)
        if kind == "per_tensor":
            e = np.full_like(e, e.max())
        q = rnd(blk * np.ldexp(1.0, -e)[..., None])
        if kind == "block_16":
            return q.reshape(x.shape), e[..., ::2]
        return q.reshape(x.shape), e
    return mx_quantize


@pytest.mark.parametrize("kind", ["ceil_log2", "emax_plus_one", "emax_minus_one", "per_tensor", "block_16"])
def test_mx_quantize_mutations_are_caught(monkeypatch, kind):
    monkeypatch.setattr(O, "mx_quantize", _mx_variant(kind))
    assert some_pin_fails()


def test_quantising_the_wrong_operand_is_caught(monkeypatch):
    monkeypatch.setattr(O, "mx_linear", lambda a, w_q, w_e: O.mx_dequantize(w_q, w_e) @ np.asarray(a, np.float64))
    assert some_pin_fails()


def test_unquantised_expert_hidden_is_caught(monkeypatch):
    orig = O.swiglu_ffn
    monkeypatch.setattr(O, "swiglu_ffn", lambda b, wg, wu, wd, hidden_in=None: orig(b, wg, wu, wd, None))
    assert some_pin_fails()


def test_activation_trace_and_override_hooks_change_no_arithmetic():
    """The bookkeeping hooks of the low-bit model (act_trace records every value about to be block-quantised;
    act_override substitutes given vectors for the oracle's own quantised ones; layers= applies a subset of the stack)
    are inert: tracing changes nothing, overriding every stage with the oracle's OWN quantised value reproduces the
    plain run bit for bit, walking the layers one at a time equals walking them together, and overriding one stage with
    a different vector does change the result (the hook is really consulted)."""
    s = synth.ModelShape(**{**SMALL.__dict__, "ffn_hidden": 64})      # every K a multiple of 32
    w = small_weights(shape=s)
    toks = synth.token_ids((1, 6), s.vocab, 5)[0]
    plain = O.PLTOracle(oshape(s), w, kv_bf16=True, w_mx=True)
    plain.clp_prefill(list(toks), 8)
    ref = np.stack(plain.trace)

    traced = O.PLTOracle(oshape(s), w, kv_bf16=True, w_mx=True)
    traced.act_trace = []; traced.layer_trace = []
    traced.clp_prefill(list(toks), 8)
    assert np.array_equal(np.stack(traced.trace), ref)
    assert len(traced.act_trace) == len(toks) * s.n_loops * s.n_layers * 4
    assert sorted({st for (_, _, st, _) in traced.act_trace}) == [0, 1, 2, 3]

    # the last position again, layer by layer, every stage overridden with the oracle's own quantised value
    p = len(toks) - 1
    mine = {}
    for (l, m, st, t) in traced.act_trace[-s.n_loops * s.n_layers * 4:]:
        mine[(l, m, st)] = O.mx_dequantize(*O.mx_quantize(t, "e4m3"))
    x_in = {(l, m): a for (l, m, pp, a, b) in traced.layer_trace if pp == p}
    x_out = {(l, m): b for (l, m, pp, a, b) in traced.layer_trace if pp == p}
    traced.act_override = mine
    for l in range(1, s.n_loops + 1):
        x = x_in[(l, 0)]
        for m in range(s.n_layers):
            x = traced.f(x, p, l, traced.kv, layers=[m])
            assert np.array_equal(x, x_out[(l, m)]), (l, m)
    # a different vector at one stage moves the output
    moved = dict(mine); moved[(1, 0, 3)] = mine[(1, 0, 3)] * 1.25
    traced.act_override = moved
    assert not np.array_equal(traced.f(x_in[(1, 0)], p, 1, traced.kv, layers=[0]), x_out[(1, 0)])
