"""The pins must be sharp: plant plausible mistakes in the oracle (on the CPU) and check that
at least one pin fails for each."""
import math

import numpy as np
import pytest

from oracle import plt_oracle as O
from tests import test_oracle_pins as P

PINS = [P.test_L1_equals_textbook_decoder,
        lambda: P.test_plt_forward_equals_token_parallel_formulation(3, 3, False),
        lambda: P.test_clp_equals_sequential(3, 4),
        P.test_gate_extremes_and_midpoint, P.test_brute_force_tiny, P.test_window_bounds_by_mask,
        P.test_full_window_open_gate_is_plain_attention, P.test_softmax_invariants,
        P.test_causality_and_shift_direction, P.test_vanilla_loop_equals_stacked_textbook]


def some_pin_fails():
    for pin in PINS:
        try:
            pin()
        except AssertionError:
            return True
    return False


def test_pins_pass_unmutated():
    assert not some_pin_fails()


def _gate_swapped(y_local, y_global, z):
    g = 1.0 / (1.0 + math.exp(-float(z)))
    return (1 - g) * np.asarray(y_local) + g * np.asarray(y_global)


def _attend_wrong_scale(q, K, V):
    s = np.asarray(K, np.float64) @ np.asarray(q, np.float64) / q.shape[-1]
    e = np.exp(s - s.max())
    return (e / e.sum()) @ np.asarray(V, np.float64)


def _rope_wrong_sign(x, p, theta):
    x = np.asarray(x, np.float64); D = x.shape[-1]; h = D // 2
    ang = p * theta ** (-2.0 * np.arange(h) / D)
    c, s = np.cos(ang), np.sin(ang)
    return np.concatenate([x[..., :h] * c + x[..., h:] * s, x[..., h:] * c + x[..., :h] * s], -1)


def _rope_interleaved(x, p, theta):
    x = np.asarray(x, np.float64); D = x.shape[-1]; h = D // 2
    ang = p * theta ** (-2.0 * np.arange(h) / D)
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(x)
    out[..., 0::2] = x[..., 0::2] * c - x[..., 1::2] * s
    out[..., 1::2] = x[..., 1::2] * c + x[..., 0::2] * s
    return out


def _norm_no_eps_mean(x, gain, eps):
    x = np.asarray(x, np.float64)
    return x / np.sqrt(np.sum(x * x, -1, keepdims=True) + eps) * np.asarray(gain, np.float64)


@pytest.mark.parametrize("name,repl", [("gate_merge", _gate_swapped), ("softmax_attend", _attend_wrong_scale),
                                       ("rope", _rope_wrong_sign), ("rope", _rope_interleaved),
                                       ("rmsnorm", _norm_no_eps_mean)])
def test_function_mutations_are_caught(monkeypatch, name, repl):
    monkeypatch.setattr(O, name, repl)
    assert some_pin_fails()


def test_window_off_by_one_is_caught(monkeypatch):
    def get_local(self, l, m, p, w):
        ks, vs = self.loc[(l, m)]
        lo = max(0, p - w)
        return np.stack(ks[lo:p + 1]), np.stack(vs[lo:p + 1])
    monkeypatch.setattr(O.FullHistoryKV, "get_local", get_local)
    assert some_pin_fails()


def test_ring_slot_mistake_is_caught(monkeypatch):
    def put_local(self, l, m, p, k, v, w):
        self.kr[l - 2, m, (p + 1) % w] = self._store(k); self.vr[l - 2, m, (p + 1) % w] = self._store(v)
    monkeypatch.setattr(O.RingKV, "put_local", put_local)
    assert some_pin_fails()


def test_exclusive_global_extent_is_caught(monkeypatch):
    orig = O.FullHistoryKV.get_global

    def get_global(self, cache_id, m, p):
        ks, vs = self.glob[(cache_id, m)]
        n = max(p, 1)
        return np.stack(ks[:n]), np.stack(vs[:n])
    monkeypatch.setattr(O.FullHistoryKV, "get_global", get_global)
    assert some_pin_fails()


def test_missing_shift_is_caught(monkeypatch):
    def seq_forward(self, tokens):
        s = self.s; n = len(tokens); kv = O.FullHistoryKV(self._store)
        E = np.stack([self.embed(t) for t in tokens]); H = np.zeros((s.n_loops, n, s.d_model))
        for p in range(n):
            H[0, p] = self.f(E[p], p, 1, kv)
        for l in range(2, s.n_loops + 1):
            for p in range(n):
                H[l - 1, p] = self.f(E[p] + H[l - 2, p], p, l, kv)      # no right shift
        return H, np.stack([self.logits(H[-1, p]) for p in range(n)])
    monkeypatch.setattr(O.PLTOracle, "seq_forward", seq_forward)
    assert some_pin_fails()


def _e4m3_truncating(x):
    a = np.clip(np.asarray(x, np.float64), -448.0, 448.0)
    _, ex = np.frexp(np.abs(a))
    step = np.ldexp(1.0, np.maximum(ex - 1, -6) - 3)
    return np.sign(a) * np.floor(np.abs(a) / step) * step


def _e4m3_no_subnormals(x):
    a = np.clip(np.asarray(x, np.float64), -448.0, 448.0)
    _, ex = np.frexp(np.abs(a))
    step = np.ldexp(1.0, ex - 1 - 3)
    return np.sign(a) * np.rint(np.abs(a) / step) * step


def _e4m3_wrong_max(x):
    a = np.clip(np.asarray(x, np.float64), -480.0, 480.0)
    _, ex = np.frexp(np.abs(a))
    step = np.ldexp(1.0, np.maximum(ex - 1, -6) - 3)
    return np.sign(a) * np.rint(np.abs(a) / step) * step


@pytest.mark.parametrize("repl", [_e4m3_truncating, _e4m3_no_subnormals, _e4m3_wrong_max])
def test_e4m3_mutations_are_caught(monkeypatch, repl):
    monkeypatch.setattr(O, "e4m3_round", repl)
    with pytest.raises(AssertionError):
        P.test_e4m3_round_matches_torch_and_the_format()
