"""Parity at the benchmark's full sizes, in the launch configuration bench.py times, on sampled
sequences (sequences of a batch are independent, so the oracle checks one at a time).

Two comparisons per decode step.  End to end: the step's logits at the stated bf16 bar of 2e-2 max-abs.  Per layer,
teacher-forced: every layer of the device is fed the ORACLE's input of that layer for the sampled sequences
(plt_debug_layer) and its output rows are held to the same 2e-2 max-abs, so that a defect of a few 1e-2 in any
single layer's residual, norm, attention or feed-forward path fails, which the end-to-end hidden state -- about
0.2 off on values of magnitude 50 after 24 layers of bf16 roundings -- could not show.  The accumulated drift of the
free-running hidden state is printed, labelled as accumulated, and only sanity-bounded."""
import ctypes as C

import numpy as np
import pytest
import torch

import bench
from oracle import plt_oracle as O
from paper_2510_24824_amd import binding as B, synth
from tests.helpers import lively_weights, oshape

pytestmark = pytest.mark.gpu


def oracle_step(shape, cfg, weights_host, exports, carry, token, pos):
    fp8 = cfg.kv_dtype == B.PLT_FP8_E4M3
    osh = O.OracleShape(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim,
                        shape.ffn_hidden, shape.vocab, cfg.n_loops, cfg.window, shape.rope_theta, shape.norm_eps,
                        shape.tie_embeddings, n_experts=cfg.n_experts, top_k=cfg.top_k)
    orc = O.PLTOracle(osh, weights_host, kv_bf16=not fp8, kv_fp8=fp8)
    orc.kv = O.RingKV(orc._store, osh, pos + 1)
    for m, e in enumerate(exports):
        orc.kv.ks[m, :pos] = e["k_share"].transpose(1, 0, 2); orc.kv.vs[m, :pos] = e["v_share"].transpose(1, 0, 2)
        for l in range(cfg.n_loops - 1):
            orc.kv.kr[l, m] = e["k_ring"][l].transpose(1, 0, 2); orc.kv.vr[l, m] = e["v_ring"][l].transpose(1, 0, 2)
    orc.carry = carry.astype(np.float64).copy(); orc.pos = pos; orc.trace = []
    orc.layer_trace = []
    nxt, lg = orc.clp_decode_step(int(token))
    oracle_step.route_margins = list(orc.route_margins)     # mixture-of-experts models: the step's routing gaps
    # the step's layer inputs / outputs [L, layers, d] (the oracle walks loop by loop, layer by layer)
    L, nl = cfg.n_loops, shape.n_layers
    x_in = np.zeros((L, nl, shape.d_model)); x_out = np.zeros_like(x_in)
    assert len(orc.layer_trace) == L * nl
    for (l, m, p, a, b) in orc.layer_trace:
        assert p == pos
        x_in[l - 1, m] = a; x_out[l - 1, m] = b
    oracle_step.layer_in, oracle_step.layer_out = x_in, x_out
    return nxt, lg, orc.trace[-1]


ROUTING_NOISE = 4e-3        # bf16 storage of the normed row moves a router logit by about 2e-3
ACCUMULATED_DRIFT_SANITY = 5e-2     # free-running hidden state after all layers, relative to its largest entry


def per_layer_teacher_forced(kv, shape, cfg, pos, layer_io, tol=2e-2, skip=None):
    """layer_io: {sequence: (x_in [L, layers, d], x_out [L, layers, d])} from the oracle.  Feeds every layer of the
    device the oracle's layer input for those sequences (zeros for the others, whose rows are not looked at) at
    position pos and returns the largest |device - oracle| over the sampled rows per layer; asserts each <= tol.
    skip(seq, loop row, layer) -> True leaves that row of that layer out (used where an integer decision inside the
    layer -- the experts chosen -- is within rounding reach and differs)."""
    Bn, L = kv.batch, cfg.n_loops
    worst = []
    for m in range(shape.n_layers):
        kv.set_position(pos)
        xin = np.zeros((Bn, L, shape.d_model), np.float32)
        for b, (x_in, _) in layer_io.items():
            xin[b] = x_in[:, m]
        out = kv.debug_layer(m, xin)
        assert kv.position == pos
        e = 0.0
        for b, (x_in, x_out) in layer_io.items():
            for l in range(L):
                if skip is not None and skip(b, l, m):
                    continue
                # the float32 copy of the input is what both sides continue from
                ref = x_out[l, m] - x_in[l, m] + xin[b, l].astype(np.float64)
                e = max(e, float(np.max(np.abs(out[b, l] - ref))))
        worst.append(e)
    print("per-layer teacher-forced max-abs:", " ".join(f"{e:.1e}" for e in worst))
    assert max(worst) <= tol, (int(np.argmax(worst)), max(worst))
    return worst


@pytest.mark.parametrize("kv_dtype,shape", [(0, synth.PLT_1P3B), (B.PLT_FP8_E4M3, synth.PLT_1P3B), (0, synth.PLT_DENSE_GQA)],
                         ids=["1p3b-bf16kv", "1p3b-e4m3kv", "dense-gqa-32q8kv"])
def test_decode_step_1p3b_L2_batch64_ctx2048_sampled(kv_dtype, shape):
    """The headline workload: 24 layers, d=2048, 16x128 heads, FFN 5632, vocab 32000, L=2, w=64,
    batch 64, 2048-token context built by plt_prefill; sequences 0 and 41 checked against the oracle.
    Also with e4m3 caches (the oracle then rounds the new position's K and V to e4m3 as well), and on
    the paper's open-source dense shape (16 layers, FFN 16384, 32 query / 8 kv heads of 64)."""
    Bn, N = 64, 2048
    pos = N - 1
    cfg = B.make_config(shape, dtype=B.PLT_BF16, n_loops=2, window=64, kv_dtype=kv_dtype)
    blob = bench.fill_weights_on_device(B, cfg, bench.SEED)
    model = B.Model(cfg, blob)
    kv = B.KV(model, Bn, N)
    g = torch.Generator(device="cuda"); g.manual_seed(bench.SEED + 1)
    prompt = torch.randint(0, shape.vocab, (Bn, pos), generator=g, device="cuda", dtype=torch.int32)
    nxt, _ = kv.prefill(prompt, want_logits=False)
    sample = [0, 41]
    state = {b: ([kv.export(b, m, pos) for m in range(shape.n_layers)], kv.get_carry()[b], int(nxt[b].item())) for b in sample}
    n1, lg1 = kv.decode_step(nxt.clone())
    hidden = kv.get_hidden()
    wh = bench.weights_to_host(B, cfg, blob)
    layer_io = {}
    for b in sample:
        exports, carry, token = state[b]
        o_next, o_lg, o_hid = oracle_step(shape, cfg, wh, exports, carry, token, pos)
        layer_io[b] = (oracle_step.layer_in, oracle_step.layer_out)
        err = float(np.max(np.abs(lg1[b].float().cpu().numpy() - o_lg)))
        abs_h = float(np.max(np.abs(hidden[b] - o_hid)))
        rel_h = abs_h / float(np.max(np.abs(o_hid)))
        print(f"seq {b}: logits max-abs {err:.3e}; accumulated hidden drift after {shape.n_layers} layers {abs_h:.3e} abs = {rel_h:.3e} of the "
              f"largest entry (reported, not the parity bar); margin {np.sort(o_lg)[-1] - np.sort(o_lg)[-2]:.3e}")
        assert err <= 2e-2, err
        assert rel_h <= ACCUMULATED_DRIFT_SANITY, rel_h
        if np.sort(o_lg)[-1] - np.sort(o_lg)[-2] > 4e-2:
            assert int(n1[b].item()) == o_next
    # The stated bar belongs to the 1.3B shape.  A projection's rounding error grows with the square root of its
    # contraction length (independent bf16 roundings of its inputs), so the shape with the 16384-wide feed-forward
    # gets the same bar scaled by sqrt(16384 / 5632) (measured: 1.4e-2 .. 2.1e-2 per layer against 0.8e-2 .. 1.3e-2).
    tol = 2e-2 * max(1.0, (shape.ffn_hidden / synth.PLT_1P3B.ffn_hidden) ** 0.5)
    per_layer_teacher_forced(kv, shape, cfg, pos, layer_io, tol=tol)
    kv.close(); model.close()


def test_decode_step_L4_w128_ctx8192_sampled():
    """The long-context shape (L=4, window 128, 8192-token shared KV per sequence) at batch 2, state
    built by plt_prefill of 8191 tokens; one sequence's decode step is recomputed by the oracle."""
    shape = synth.PLT_1P3B
    Bn, N, L, w = 2, 8192, 4, 128
    pos = N - 1
    cfg = B.make_config(shape, dtype=B.PLT_BF16, n_loops=L, window=w)
    blob = bench.fill_weights_on_device(B, cfg, bench.SEED)
    model = B.Model(cfg, blob)
    kv = B.KV(model, Bn, N)
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    prompt = torch.randint(0, shape.vocab, (Bn, pos), generator=g, device="cuda", dtype=torch.int32)
    nxt, _ = kv.prefill(prompt, want_logits=False)
    b = 1
    exports = [kv.export(b, m, pos) for m in range(shape.n_layers)]
    carry = kv.get_carry()
    tok = nxt.clone()
    n1, lg1 = kv.decode_step(tok)
    hidden = kv.get_hidden()
    wh = bench.weights_to_host(B, cfg, blob)
    o_next, o_lg, o_hid = oracle_step(shape, cfg, wh, exports, carry[b], int(tok[b].item()), pos)
    err = float(np.max(np.abs(lg1[b].float().cpu().numpy() - o_lg)))
    rel_h = float(np.max(np.abs(hidden[b] - o_hid)) / np.max(np.abs(o_hid)))
    per_row = [float(np.max(np.abs(hidden[b, l] - o_hid[l])) / np.max(np.abs(o_hid[l]))) for l in range(L)]
    print(f"logits max-abs {err:.3e} (max |logit| {np.max(np.abs(o_lg)):.2f}); accumulated hidden drift {rel_h:.3e} of the largest "
          f"entry (reported); per row {per_row}; max |hidden| {np.max(np.abs(o_hid)):.1f}")
    assert err <= 2e-2 and rel_h <= ACCUMULATED_DRIFT_SANITY, (err, rel_h)
    per_layer_teacher_forced(kv, shape, cfg, pos, {b: (oracle_step.layer_in, oracle_step.layer_out)})
    kv.set_position(pos + 1)
    # batch independence: the same sequence alone in a batch of 1 gives the same logits (the split
    # count of the attention kernel differs, so agreement is to rounding, not bit for bit)
    kv1 = B.KV(model, 1, N)
    for m in range(shape.n_layers):
        e = exports[m]
        kv1.import_(0, m, pos, e["k_share"], e["v_share"], e["k_ring"], e["v_ring"])
    kv1.set_carry(carry[b:b + 1]); kv1.set_position(pos)
    _, lg_solo = kv1.decode_step(tok[b:b + 1].clone())
    assert float(torch.max(torch.abs(lg_solo[0] - lg1[b]))) <= 1e-2
    kv1.close(); kv.close(); model.close()


def test_decode_step_160_rows_sampled():
    """Batch 40 x L = 4 = 160 rows per step: the row count (129..256) at which the gate/up projection
    runs as one fused-SwiGLU tile per 32 output columns; short context so that the oracle is quick."""
    shape = synth.PLT_1P3B
    Bn, N, L, w = 40, 300, 4, 64
    pos = N - 1
    cfg = B.make_config(shape, dtype=B.PLT_BF16, n_loops=L, window=w)
    blob = bench.fill_weights_on_device(B, cfg, bench.SEED)
    model = B.Model(cfg, blob)
    kv = B.KV(model, Bn, N)
    g = torch.Generator(device="cuda"); g.manual_seed(11)
    prompt = torch.randint(0, shape.vocab, (Bn, pos), generator=g, device="cuda", dtype=torch.int32)
    nxt, _ = kv.prefill(prompt, want_logits=False)
    b = 23
    exports = [kv.export(b, m, pos) for m in range(shape.n_layers)]
    carry = kv.get_carry()
    tok = nxt.clone()
    n1, lg1 = kv.decode_step(tok)
    hidden = kv.get_hidden()
    wh = bench.weights_to_host(B, cfg, blob)
    o_next, o_lg, o_hid = oracle_step(shape, cfg, wh, exports, carry[b], int(tok[b].item()), pos)
    err = float(np.max(np.abs(lg1[b].float().cpu().numpy() - o_lg)))
    rel_h = float(np.max(np.abs(hidden[b] - o_hid)) / np.max(np.abs(o_hid)))
    print(f"logits max-abs {err:.3e}; accumulated hidden drift {rel_h:.3e} of the largest entry (reported)")
    assert err <= 2e-2 and rel_h <= ACCUMULATED_DRIFT_SANITY, (err, rel_h)
    per_layer_teacher_forced(kv, shape, cfg, pos, {b: (oracle_step.layer_in, oracle_step.layer_out)})
    kv.close(); model.close()


def test_decode_step_moe_8_of_64_batch64_ctx2048_sampled():
    """The paper's open-source mixture-of-experts recipe per layer (hidden 2048, 16 heads of 128, 64 SwiGLU
    experts of hidden 1024, 8 per token), two layers deep so that the host copy of the weights stays small;
    batch 64 x L = 2 at a 2048-token context built by plt_prefill (which routes 16k rows per chunk through the
    same grouped kernels).  Sampled sequences are recomputed by the oracle from the exported state.  A
    sequence that disagrees while its smallest routing gap in this step is within reach of bf16 rounding is
    reported and its end-to-end comparison not asserted; at least two of the three samples must agree end to end, and
    every (row, layer) pair with a routing gap above that noise must agree per layer."""
    shape = bench.with_layers(synth.PLT_MOE_1B7B, 2)
    Bn, N = 64, 2048
    pos = N - 1
    cfg = B.make_config(shape, dtype=B.PLT_BF16, n_loops=2, window=64)
    blob = bench.fill_weights_on_device(B, cfg, bench.SEED)
    model = B.Model(cfg, blob)
    kv = B.KV(model, Bn, N)
    g = torch.Generator(device="cuda"); g.manual_seed(bench.SEED + 3)
    prompt = torch.randint(0, shape.vocab, (Bn, pos), generator=g, device="cuda", dtype=torch.int32)
    nxt, _ = kv.prefill(prompt, want_logits=False)
    sample = [0, 29, 63]
    state = {b: ([kv.export(b, m, pos) for m in range(shape.n_layers)], kv.get_carry()[b], int(nxt[b].item())) for b in sample}
    n1, lg1 = kv.decode_step(nxt.clone())
    hidden = kv.get_hidden()
    wh = bench.weights_to_host(B, cfg, blob)
    clear = 0
    layer_io, gaps = {}, {}
    for b in sample:
        exports, carry, token = state[b]
        o_next, o_lg, o_hid = oracle_step(shape, cfg, wh, exports, carry, token, pos)
        layer_io[b] = (oracle_step.layer_in, oracle_step.layer_out)
        gaps[b] = np.array(oracle_step.route_margins).reshape(cfg.n_loops, shape.n_layers)    # the oracle walks loop by loop
        gap = float(gaps[b].min())
        err = float(np.max(np.abs(lg1[b].float().cpu().numpy() - o_lg)))
        rel_h = float(np.max(np.abs(hidden[b] - o_hid)) / np.max(np.abs(o_hid)))
        print(f"seq {b}: smallest routing gap {gap:.3e}; logits max-abs {err:.3e}; accumulated hidden drift {rel_h:.3e} of the largest entry")
        ok = err <= 2e-2 and rel_h <= ACCUMULATED_DRIFT_SANITY
        if not ok and gap < ROUTING_NOISE:      # router logits are ~N(0, 0.9); bf16 activations move them by ~2e-3
            print(f"seq {b}: a routing decision of this step is within rounding reach; the end-to-end comparison of this sequence is not asserted")
            continue
        assert ok, (b, err, rel_h, gap)        # a disagreement with every gap above the noise is a failure
        clear += 1
    assert clear >= 2
    # per layer, from the oracle's layer input: every row of every layer whose routing gap is above the noise must
    # match at the bf16 bar (a row within reach of the noise may legitimately evaluate a different expert)
    n_skipped = sum(int(np.sum(g < ROUTING_NOISE)) for g in gaps.values())
    per_layer_teacher_forced(kv, shape, cfg, pos, layer_io, skip=lambda b, l, m: gaps[b][l, m] < ROUTING_NOISE)
    print(f"per-layer comparison left out {n_skipped} of {len(sample) * cfg.n_loops * shape.n_layers} (row, layer) pairs with a routing gap below {ROUTING_NOISE}")
    assert n_skipped <= 2
    kv.close(); model.close()


def _untile(t):
    """Inverse of binding.moe_tile_weights for one matrix: blob strip order -> logical [N, K]."""
    N, K = t.shape
    return np.ascontiguousarray(t.reshape(N // 16, K // 32, 4, 16, 8).transpose(0, 3, 1, 2, 4)).reshape(N, K)


def test_moe_ffn_one_prefill_chunk_16384_rows_sampled():
    """The mixture-of-experts feed-forward alone at the size of one prefill chunk of the paper's 8-of-64 recipe
    (16384 rows of 2048, 64 SwiGLU experts of hidden 1024, 8 per row): the router on the matrix cores, the stable
    sort of 131072 (row, slot) pairs over many workgroups, both grouped GEMMs on 256 x 256 tiles.  The weights are
    drawn on the device directly in the blob's strip order (a random matrix in any order is a random matrix) and
    un-permuted on the host for the experts the sampled rows select; the oracle recomputes those rows."""
    from tests.test_gpu_moe import _bf16_bound
    R, d, F, E, k = 16384, 2048, 1024, 64, 8
    g = torch.Generator(device="cuda"); g.manual_seed(bench.SEED + 21)
    bf = torch.bfloat16
    a = torch.randn(R, d, generator=g, device="cuda").to(bf)
    router = (torch.randn(E, d, generator=g, device="cuda") * 0.05).to(bf)
    gu = (torch.randn(E, 2 * F, d, generator=g, device="cuda") * 0.02).to(bf)      # strip order
    dn = (torch.randn(E, d, F, generator=g, device="cuda") * 0.02).to(bf)          # strip order
    y = torch.empty(R, d, dtype=torch.float32, device="cuda")
    sel_e = torch.empty(R, k, dtype=torch.int32, device="cuda")
    sel_p = torch.empty(R, k, dtype=torch.float32, device="cuda")
    lib = B.lib()
    nb = lib.plt_moe_scratch_bytes(B.PLT_BF16, R, d, F, E, k)
    assert nb > 0, lib.plt_last_error().decode()
    scratch = torch.empty(nb, dtype=torch.uint8, device="cuda")
    rc = lib.plt_moe_ffn(B.PLT_BF16, R, d, F, E, k, a.data_ptr(), router.data_ptr(), gu.data_ptr(), dn.data_ptr(),
                         y.data_ptr(), sel_e.data_ptr(), sel_p.data_ptr(), scratch.data_ptr(), nb,
                         torch.cuda.current_stream().cuda_stream)
    assert rc == 0, lib.plt_last_error().decode()
    torch.cuda.synchronize()
    se = sel_e.cpu().numpy(); sp = sel_p.cpu().numpy()
    # every row: k distinct experts, probabilities in decreasing order; the lists cover all R * k pairs
    assert np.all(np.sort(se, axis=1)[:, 1:] != np.sort(se, axis=1)[:, :-1]) and np.all(np.diff(sp, axis=1) <= 0)
    counts = np.bincount(se.reshape(-1), minlength=E)
    print(f"rows per expert min/mean/max {counts.min()}/{counts.mean():.0f}/{counts.max()}")
    router_h = router.float().cpu().numpy()
    compared = 0
    for r in (0, 255, 256, 4099, 8191, 12345, 16382, 16383):    # first / last rows of row tiles and chunks, some inside
        b = a[r].float().cpu().numpy()
        ids, p, margin = O.moe_route(b, router_h, k)
        if margin < 1e-4:                       # float and float64 logits may order the boundary pair differently
            print(f"row {r}: routing gap {margin:.3e}: not compared")
            continue
        assert list(se[r]) == list(ids), (r, se[r], ids, margin)
        assert np.max(np.abs(sp[r] - p)) <= 1e-5
        W = {"w_gate": {}, "w_up": {}, "w_down": {}}
        ref = np.zeros(d)
        for e, pe in zip(ids, p):
            gate_up = _untile(gu[e].float().cpu().numpy())
            W["w_gate"][e], W["w_up"][e], W["w_down"][e] = gate_up[:F], gate_up[F:], _untile(dn[e].float().cpu().numpy())
            ref += pe * O.swiglu_ffn(b, W["w_gate"][e], W["w_up"][e], W["w_down"][e], None)
        err = np.abs(y[r].cpu().numpy() - ref)
        tol = _bf16_bound(b, W, ids, p) + 1e-5 * max(float(np.max(np.abs(ref))), 1.0)    # as in tests/test_gpu_moe.py
        print(f"row {r}: routing gap {margin:.3e}; max |y| {np.max(np.abs(ref)):.3e}; max err {err.max():.3e}")
        assert np.all(err <= tol) and err.max() <= 2e-2, (r, float(err.max()))
        compared += 1
    assert compared >= 5


@pytest.mark.parametrize("kv_dtype", [0, B.PLT_FP8_E4M3], ids=["bf16kv", "e4m3kv"])
def test_prefill_4x8192_L3_equals_shorter_prefill_plus_decode_steps(kv_dtype):
    """The prefill workload bench.py times (4 prompts of 8192 tokens, L = 3, window 64, the 1.3B widths; two layers
    deep) cannot be walked by the position-by-position oracle in seconds, so it is checked through a property that
    holds at any size [Alg. 1 l.1-3: the prompt is consumed by the same micro-batch rule as decoding]: the prefill
    of all n tokens must leave the state that the prefill of the first n - 37 tokens followed by 37 teacher-forced
    decode steps leaves -- and those decode steps are checked against the oracle at full size above.  Compared:
    the last position's logits, the carry, and for sampled sequences both layers' shared K/V (positions both paths
    took through the prefill kernels: identical; the last 37: equal to bf16 rounding, or to one e4m3 step = 1/16 of
    the largest entry for e4m3 caches) and rings."""
    shape = bench.with_layers(synth.PLT_1P3B, 2)
    Bn, n, m = 4, 8192, 37
    cfg = B.make_config(shape, dtype=B.PLT_BF16, n_loops=3, window=64, kv_dtype=kv_dtype)
    kv_tol = 0.07 if kv_dtype == B.PLT_FP8_E4M3 else 2e-2
    blob = bench.fill_weights_on_device(B, cfg, bench.SEED)
    model = B.Model(cfg, blob)
    g = torch.Generator(device="cuda"); g.manual_seed(bench.SEED + 31)
    tokens = torch.randint(0, shape.vocab, (Bn, n), generator=g, device="cuda", dtype=torch.int32)
    kv_a = B.KV(model, Bn, n + 1)
    next_a, lg_a = kv_a.prefill(tokens)
    next_a = next_a.cpu().numpy().copy(); lg_a = lg_a.float().cpu().numpy().copy()
    kv_b = B.KV(model, Bn, n + 1)
    kv_b.prefill(tokens[:, :n - m].contiguous(), want_logits=False)
    for i in range(m):
        next_b, lg_b = kv_b.decode_step(tokens[:, n - m + i].contiguous())
    next_b = next_b.cpu().numpy(); lg_b = lg_b.float().cpu().numpy()
    top = float(np.max(np.abs(lg_a)))
    d_lg = float(np.max(np.abs(lg_a - lg_b)))
    ca, cb = kv_a.get_carry(), kv_b.get_carry()
    d_c = float(np.max(np.abs(ca - cb)) / np.max(np.abs(ca)))
    print(f"logits: max |.| {top:.3f}, max difference {d_lg:.3e}; carry: max relative difference {d_c:.3e}")
    # both paths round every stored activation to bf16 (2^-8 relative) and differ in accumulation order only; each
    # is within 1 % of the largest logit of the exact result (the bar of the oracle comparisons), so the two are
    # within 2 % of each other
    assert d_lg <= 2e-2 * top and d_c <= 2e-2
    margin = np.sort(lg_a, axis=1)
    for b in range(Bn):
        if margin[b, -1] - margin[b, -2] > 4e-2 * top:
            assert next_a[b] == next_b[b], (b, next_a[b], next_b[b])
    for b in (0, Bn - 1):
        for layer in range(shape.n_layers):
            ea, eb = kv_a.export(b, layer, n), kv_b.export(b, layer, n)
            for name in ("k_share", "v_share"):
                assert np.array_equal(ea[name][:, :n - m], eb[name][:, :n - m]), (b, layer, name)
                scale = float(np.max(np.abs(ea[name][:, n - m:])))
                diff = float(np.max(np.abs(ea[name][:, n - m:] - eb[name][:, n - m:])))
                assert diff <= kv_tol * scale, (b, layer, name, diff, scale)
            for name in ("k_ring", "v_ring"):
                scale = float(np.max(np.abs(ea[name])))
                diff = float(np.max(np.abs(ea[name] - eb[name])))
                assert diff <= kv_tol * scale, (b, layer, name, diff, scale)
            print(f"seq {b} layer {layer}: shared K/V identical below position {n - m}; last {m} and rings within {kv_tol:.0%} of the largest entry")
    kv_a.close(); kv_b.close(); model.close()


def test_decode_step_L4_w128_ctx8192_batch128_sampled():
    """One GPU's share of the long-context configuration (L = 4, window 128, 8192-token shared KV, batch 128:
    206 GB of shared K/V + 9.7 GB of windows resident), in the launch configuration bench.py times: one workgroup per
    (sequence, kv head) stream, no split.  State built by plt_prefill of 128 x 8191 tokens; one sampled sequence's
    decode step is recomputed by the oracle from the exported state: logits end to end, every layer teacher-forced."""
    shape = synth.PLT_1P3B
    Bn, N, L, w = 128, 8192, 4, 128
    pos = N - 1
    cfg = B.make_config(shape, dtype=B.PLT_BF16, n_loops=L, window=w)
    blob = bench.fill_weights_on_device(B, cfg, bench.SEED)
    model = B.Model(cfg, blob)
    free = torch.cuda.mem_get_info()[0]
    need = model.kv_bytes(Bn, N)
    if need > free - (12 << 30):
        pytest.skip(f"needs {need / 2**30:.0f} GiB of KV, {free / 2**30:.0f} GiB free on this device")
    kv = B.KV(model, Bn, N)
    g = torch.Generator(device="cuda"); g.manual_seed(17)
    prompt = torch.randint(0, shape.vocab, (Bn, pos), generator=g, device="cuda", dtype=torch.int32)
    nxt, _ = kv.prefill(prompt, want_logits=False)
    b = 77
    exports = [kv.export(b, m, pos) for m in range(shape.n_layers)]
    carry = kv.get_carry()
    tok = nxt.clone()
    n1, lg1 = kv.decode_step(tok)
    hidden = kv.get_hidden()
    wh = bench.weights_to_host(B, cfg, blob)
    o_next, o_lg, o_hid = oracle_step(shape, cfg, wh, exports, carry[b], int(tok[b].item()), pos)
    err = float(np.max(np.abs(lg1[b].float().cpu().numpy() - o_lg)))
    rel_h = float(np.max(np.abs(hidden[b] - o_hid)) / np.max(np.abs(o_hid)))
    print(f"seq {b} of {Bn}: logits max-abs {err:.3e}; accumulated hidden drift {rel_h:.3e} of the largest entry (reported)")
    assert err <= 2e-2 and rel_h <= ACCUMULATED_DRIFT_SANITY, (err, rel_h)
    if np.sort(o_lg)[-1] - np.sort(o_lg)[-2] > 4e-2:
        assert int(n1[b].item()) == o_next
    per_layer_teacher_forced(kv, shape, cfg, pos, {b: (oracle_step.layer_in, oracle_step.layer_out)})
    kv.close(); model.close()


@pytest.mark.parametrize("heads,kv_dtype,mode", [((2, 1, 128), 0, B.PLT_MODE_CLP), ((2, 1, 128), B.PLT_FP8_E4M3, B.PLT_MODE_CLP),
                                                 ((4, 2, 64), 0, B.PLT_MODE_CLP), ((2, 1, 128), 0, B.PLT_MODE_CLP_SHARE_ONLY)],
                         ids=["heads128-bf16kv", "heads128-e4m3kv", "heads64-bf16kv", "heads128-bf16kv-share-only"])
def test_prefill_4x8192_L3_narrow_model_against_oracle(heads, kv_dtype, mode):
    """The long-prompt prefill path itself against the oracle: 4 prompts of 8192 tokens at L = 3, window 64 (the
    prefill workload's batch, length, loops and window) on a narrow model (1 layer, d = 128, 2 query heads / 1 kv
    head of 128) that the position-by-position oracle walks in seconds.  8192 positions per sequence make plt_prefill
    run two chunks of two sequences (16384 rows each), 64 query tiles of 128 rows and up to 128 key steps of 64 per
    sequence.  For one sequence of each chunk the oracle consumes the same prompt by Alg. 1's micro-batch rule (equal
    to Alg. 2's loop-major pass: pinned at 1e-10 in the oracle's own tests) and is compared with the device's: shared
    K/V at EVERY position (the keys of layer 0 depend on the embedding only, the point is the cache indexing of both
    chunks), windows, carried states H^(1), H^(2) of the last position, last-position logits; and, for the sequence
    of the last chunk, the residual rows H^(3)[p] and H^(2)[p] of every position p, which plt_prefill leaves in its
    workspace (rows of the last chunk, at offset 0 and at the next multiple of 256 bytes after them).
    The QKV projection of such a chunk (16384 rows x 512 columns: 128 tiles) carries RoPE, the gate logit and the cache
    appends as its epilogue, so the every-position cache comparison is that epilogue's check; also with heads of 64
    (two heads per wave), in the KV-share-only ablation mode (non-first loops append nothing and have no gate) and with
    e4m3 caches (stored values: the oracle's code or its neighbour, i.e. within one step
    = 2^-3 of the value, plus the bf16 bar on the pre-rounding values)."""
    Hq, Hkv, D = heads
    fp8 = kv_dtype == B.PLT_FP8_E4M3
    shape = synth.ModelShape(n_layers=1, d_model=128, n_heads=Hq, n_kv_heads=Hkv, head_dim=D, ffn_hidden=256,
                             vocab=512, n_loops=3, window=64)
    Bn, n, L = 4, 8192, 3
    weights = lively_weights(shape, 21, bf16=True, std=0.05)
    share_only = mode == B.PLT_MODE_CLP_SHARE_ONLY
    cfg = B.make_config(shape, dtype=B.PLT_BF16, kv_dtype=kv_dtype, mode=mode)
    model = B.Model(cfg, B.pack_weights(cfg, weights))
    kv = B.KV(model, Bn, n + 1)
    prompts = synth.token_ids((Bn, n), shape.vocab, 22)
    nxt, lg = kv.prefill(torch.from_numpy(np.ascontiguousarray(prompts, np.int32)).cuda())
    torch.cuda.synchronize()
    nxt = nxt.cpu().numpy(); lg = lg.float().cpu().numpy()
    carry = kv.get_carry()
    d = shape.d_model
    Bc = max(1, min(Bn, 16384 // n)); rows = Bc * n
    assert Bc == 2, "two chunks of two sequences are the point of this case"
    ws = kv._ws
    x_last = ws[:rows * d * 4].view(torch.float32).reshape(Bc, n, d).cpu().numpy()          # H^(L) of the last chunk
    off = (rows * d * 4 + 255) // 256 * 256
    x_prev = ws[off:off + rows * d * 4].view(torch.float32).reshape(Bc, n, d).cpu().numpy()  # H^(L-1) of the last chunk
    wf = {k: np.asarray(v, np.float64) for k, v in weights.items() if k != "layers"}     # (conversion once, not per call)
    wf["layers"] = [{k: np.asarray(v, np.float64) for k, v in lw.items()} for lw in weights["layers"]]
    for b in (1, 3):             # last sequence of the first chunk, last sequence of the second
        orc = O.PLTOracle(oshape(shape), wf, kv_bf16=not fp8, kv_fp8=fp8, variant="clp_share_only" if share_only else "plt")
        o_next, o_lg = orc.clp_prefill(list(prompts[b]), n + 1)
        H = np.stack(orc.trace)                                   # [n, L, d]
        e_lg = float(np.max(np.abs(lg[b] - o_lg)))
        e_c = float(np.max(np.abs(carry[b] - H[n - 1, :L - 1])))
        e = kv.export(b, 0, n)
        e_ks = float(np.max(np.abs(e["k_share"] - orc.kv.ks[0, :n].transpose(1, 0, 2))))
        e_vs = float(np.max(np.abs(e["v_share"] - orc.kv.vs[0, :n].transpose(1, 0, 2))))
        e_kr = e_vr = 0.0
        if not share_only:                                       # (that mode keeps no windows)
            e_kr = float(np.max(np.abs(e["k_ring"] - orc.kv.kr[:, 0].transpose(0, 2, 1, 3))))
            e_vr = float(np.max(np.abs(e["v_ring"] - orc.kv.vr[:, 0].transpose(0, 2, 1, 3))))
        print(f"seq {b}: logits {e_lg:.2e} (max |logit| {np.max(np.abs(o_lg)):.2f}); carry {e_c:.2e} (max |H| {np.max(np.abs(H)):.2f}); "
              f"shared K {e_ks:.2e} V {e_vs:.2e}; window K {e_kr:.2e} V {e_vr:.2e}")
        # K/V: both sides round the same float value to bf16 up to float32-vs-float64 noise: equal or one bf16 step apart
        kmax = float(np.max(np.abs(orc.kv.ks[0, :n])))
        step = 2.0 ** -3 if fp8 else 2.0 ** -7        # e4m3: neighbouring codes are up to 2^-3 of the value apart
        assert max(e_ks, e_kr) <= step * kmax and max(e_vs, e_vr) <= step * float(np.max(np.abs(orc.kv.vs[0, :n])))
        if fp8:                                       # ... and all but a few per cent of the codes are the oracle's own
            same = np.mean(e["k_share"] == orc.kv.ks[0, :n].transpose(1, 0, 2).astype(np.float32))
            same_v = np.mean(e["v_share"] == orc.kv.vs[0, :n].transpose(1, 0, 2).astype(np.float32))
            print(f"seq {b}: e4m3 codes equal to the oracle's: K {same:.4f}, V {same_v:.4f}")
            assert same >= 0.94 and same_v >= 0.94
        assert e_lg <= (4e-2 if fp8 else 2e-2) and e_c <= (4e-2 if fp8 else 2e-2), (b, e_lg, e_c)
        if np.sort(o_lg)[-1] - np.sort(o_lg)[-2] > 4e-2:
            assert int(nxt[b]) == o_next
        if b >= Bn - Bc:
            i = b - (Bn - Bc)
            e3 = np.max(np.abs(x_last[i] - H[:, L - 1]), axis=1)          # per position
            e2 = np.max(np.abs(x_prev[i] - H[:, L - 2]), axis=1)
            worst3, worst2 = int(np.argmax(e3)), int(np.argmax(e2))
            print(f"seq {b}: H^(3) over all {n} positions max-abs {e3.max():.2e} (at position {worst3}); H^(2) {e2.max():.2e} (at {worst2}); "
                  f"tile and chunk borders 127/128: {e3[127]:.1e}/{e3[128]:.1e}, 63/64/65 (window): {e3[63]:.1e}/{e3[64]:.1e}/{e3[65]:.1e}, "
                  f"8191: {e3[8191]:.1e}")
            if fp8:
                # e4m3 caches: about 5 % of the stored codes are the oracle's NEIGHBOUR (the two sides' pre-rounding values
                # straddle a boundary), each such element off by a whole step = up to 2^-3 of its value.  Where few keys
                # share the softmax weight (early positions, the window border) one such V element reaches the output
                # undiluted, so over 8192 positions x 128 features the largest deviation is a flipped code's, not the
                # arithmetic's: the bar of the e4m3 model tests (4e-2, tests/test_gpu_fp8.py) must hold at all but
                # 0.2 % of the positions, and a flipped code's reach (one step of the largest V entry, ~0.125) everywhere
                frac3, frac2 = float(np.mean(e3 > 4e-2)), float(np.mean(e2 > 4e-2))
                print(f"seq {b}: positions beyond 4e-2: H^(3) {frac3:.4%}, H^(2) {frac2:.4%}")
                assert frac3 <= 2e-3 and frac2 <= 2e-3 and e3.max() <= 0.125 and e2.max() <= 0.125, (b, frac3, frac2, float(e3.max()), float(e2.max()))
            else:
                assert e3.max() <= 2e-2 and e2.max() <= 2e-2, (b, float(e3.max()), float(e2.max()))
    kv.close(); model.close()
