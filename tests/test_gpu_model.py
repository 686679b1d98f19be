"""End-to-end parity of plt_prefill / plt_decode_step (through the C ABI) with the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import plt_oracle as O
from paper_2510_24824_amd import binding as B, synth
from tests.helpers import lively_weights, oshape, with_shape

pytestmark = pytest.mark.gpu


def dev_tokens(arr):
    return torch.from_numpy(np.ascontiguousarray(arr, np.int32)).cuda()


def run_teacher_forced(shape, dtype, mode, weights, prompts, n_steps, tol, check_hidden=True, kv_dtype=0, w_dtype=0):
    """GPU consumes the oracle's token stream; logits (and hidden rows) compared at every step."""
    fp8 = kv_dtype == B.PLT_FP8_E4M3
    bf = dtype == B.PLT_BF16 and not fp8
    cfg = B.make_config(shape, dtype=dtype, mode=mode, kv_dtype=kv_dtype, w_dtype=w_dtype)
    model = B.Model(cfg, B.pack_weights(cfg, weights))
    Bn, n = prompts.shape
    kv = B.KV(model, Bn, n + n_steps + 3)
    orcs, streams, ref_logits, ref_hidden = [], [], [], []
    for b in range(Bn):
        variant = {B.PLT_MODE_CLP_SHARE_ONLY: "clp_share_only", B.PLT_MODE_CLP_OWN_KV: "clp_own_kv"}.get(mode, "plt")
        orc = O.PLTOracle(oshape(shape), weights, kv_bf16=bf, variant=variant, kv_fp8=fp8, w_mx=w_dtype == B.PLT_MXFP4)
        if mode != B.PLT_MODE_VANILLA_LOOP:
            ids, margins, lgs = orc.greedy_generate(list(prompts[b]), n_steps)
            hidden = np.stack(orc.trace)[n - 1:]                         # [n_steps+1, L, d]
        else:
            toks = list(prompts[b]); lgs = []; hid = []
            for step in range(n_steps + 1):
                H, lg = orc.vanilla_loop_forward(toks)
                lgs.append(lg[-1]); hid.append(H[-1:, -1]); toks.append(int(np.argmax(lg[-1])))
            ids = toks[n:]; lgs = np.stack(lgs); hidden = np.stack(hid)
        streams.append(ids); ref_logits.append(lgs); ref_hidden.append(hidden)
    streams = np.array(streams); ref_logits = np.stack(ref_logits); ref_hidden = np.stack(ref_hidden)
    worst = 0.0
    nxt, lg = kv.prefill(dev_tokens(prompts))
    worst = max(worst, np.max(np.abs(lg.cpu().numpy() - ref_logits[:, 0])))
    for step in range(n_steps):
        nxt, lg = kv.decode_step(dev_tokens(streams[:, step]))
        worst = max(worst, np.max(np.abs(lg.cpu().numpy() - ref_logits[:, step + 1])))
        if check_hidden:
            worst = max(worst, np.max(np.abs(kv.get_hidden() - ref_hidden[:, step + 1])))
    assert kv.position == n + n_steps
    print(f"worst abs err {worst:.3e}; max |logit| {np.max(np.abs(ref_logits)):.3f}; max |hidden| {np.max(np.abs(ref_hidden)):.3f}")
    assert worst <= tol, worst
    kv.close(); model.close()
    return worst


def test_tiny_config_greedy_ids_identical():
    """2 layers, d=256, 4 heads of 64, FFN 1024, vocab 1024, L=2, w=16, float; 64-token prompt, 32 steps."""
    shape = synth.TINY
    seed = 0
    weights = synth.make_weights(shape, seed, bf16=False)
    prompt = synth.token_ids((1, 64), shape.vocab, seed)
    orc = O.PLTOracle(oshape(shape), weights)
    ids, margins, lgs = orc.greedy_generate(list(prompt[0]), 32)
    assert min(margins) > 1e-3, "seed gives a near-tie; pick another"
    cfg = B.make_config(shape, dtype=B.PLT_F32)
    model = B.Model(cfg, B.pack_weights(cfg, weights))
    kv = B.KV(model, 1, 64 + 33)
    got, worst = [], 0.0
    nxt, lg = kv.prefill(dev_tokens(prompt))
    got.append(int(nxt.cpu()[0])); worst = max(worst, np.max(np.abs(lg.cpu().numpy()[0] - lgs[0])))
    for step in range(32):
        nxt, lg = kv.decode_step(nxt.clone())
        got.append(int(nxt.cpu()[0])); worst = max(worst, np.max(np.abs(lg.cpu().numpy()[0] - lgs[step + 1])))
    assert got == ids
    assert worst <= 1e-5, worst
    # Table 1 row 5: logical cache bytes = 2 * layers * Hkv * D * (n + (L-1) w) * 4
    assert model.kv_logical_bytes(1, 96) == O.kv_cache_bytes(oshape(shape), 96, 4)


@pytest.mark.parametrize("L,w,heads", [(3, 5, (4, 2)), (2, 16, (4, 4)), (1, 1, (4, 1)), (4, 3, (2, 2))])
def test_f32_small_models(L, w, heads):
    shape = synth.ModelShape(n_layers=2, d_model=96, n_heads=heads[0], n_kv_heads=heads[1], head_dim=64,
                             ffn_hidden=160, vocab=300, n_loops=L, window=w, tie_embeddings=(L != 3))
    weights = lively_weights(shape, 3, bf16=False, std=0.08)
    prompts = synth.token_ids((2, 11), shape.vocab, 4)
    run_teacher_forced(shape, B.PLT_F32, B.PLT_MODE_CLP, weights, prompts, 9, 2e-5)


@pytest.mark.parametrize("L,w,heads,D", [(3, 8, (4, 2), 64), (2, 64, (2, 2), 128), (1, 1, (4, 4), 64), (4, 40, (8, 2), 64)])
def test_bf16_small_models(L, w, heads, D):
    shape = synth.ModelShape(n_layers=2, d_model=128, n_heads=heads[0], n_kv_heads=heads[1], head_dim=D,
                             ffn_hidden=320, vocab=500, n_loops=L, window=w)
    weights = lively_weights(shape, 5, bf16=True, std=0.02)      # the paper-style N(0, 0.02) init
    prompts = synth.token_ids((3, 45), shape.vocab, 6)
    run_teacher_forced(shape, B.PLT_BF16, B.PLT_MODE_CLP, weights, prompts, 12, 2e-2)


@pytest.mark.parametrize("n,L,w,heads,D", [(333, 3, 40, (4, 2), 64), (200, 2, 100, (2, 2), 128), (130, 2, 64, (2, 1), 128)])
def test_bf16_prompts_of_several_key_tiles(n, L, w, heads, D):
    """Prompts longer than one workgroup's 128 query rows and than several 64-key steps, with lengths and windows
    that are no multiples of 32: the prefill attention's step ranges start and end inside 64-key steps (odd first
    32-key block of a window, last block beyond the prompt), and the state it hands to the decode steps that
    follow crosses tile boundaries.  Teacher-forced against the oracle like the small cases."""
    shape = synth.ModelShape(n_layers=2, d_model=128, n_heads=heads[0], n_kv_heads=heads[1], head_dim=D,
                             ffn_hidden=320, vocab=500, n_loops=L, window=w)
    weights = lively_weights(shape, 9, bf16=True, std=0.02)
    prompts = synth.token_ids((2, n), shape.vocab, 12)
    run_teacher_forced(shape, B.PLT_BF16, B.PLT_MODE_CLP, weights, prompts, 4, 2e-2)


@pytest.mark.parametrize("dtype,tol", [(B.PLT_F32, 2e-5), (B.PLT_BF16, 2e-2)])
def test_vanilla_loop_mode(dtype, tol):
    shape = synth.ModelShape(n_layers=2, d_model=128, n_heads=4, n_kv_heads=2, head_dim=64,
                             ffn_hidden=192, vocab=400, n_loops=3, window=8)
    weights = lively_weights(shape, 7, bf16=dtype == B.PLT_BF16, std=0.02)
    prompts = synth.token_ids((2, 9), shape.vocab, 8)
    run_teacher_forced(shape, dtype, B.PLT_MODE_VANILLA_LOOP, weights, prompts, 5, tol)


def test_state_errors_and_context_limit():
    shape = with_shape(synth.TINY, n_layers=1)
    weights = synth.make_weights(shape, 1, bf16=False)
    cfg = B.make_config(shape, dtype=B.PLT_F32)
    model = B.Model(cfg, B.pack_weights(cfg, weights))
    kv = B.KV(model, 1, 6)
    tok = dev_tokens(np.array([1]))
    with pytest.raises(B.PltError) as e:
        kv.decode_step(tok)
    assert e.value.code == -5
    with pytest.raises(B.PltError) as e:
        kv.prefill(dev_tokens(np.zeros((1, 7))))
    assert e.value.code == -3
    kv.prefill(dev_tokens(np.array([[1, 2, 3, 4, 5]])))
    kv.decode_step(tok)
    assert kv.position == 6
    with pytest.raises(B.PltError) as e:
        kv.decode_step(tok)
    assert e.value.code == -3 and kv.position == 6
    kv.close(); model.close()


def test_kv_export_import_roundtrip_and_resume():
    """Export after prefill, import into a fresh kv object, continue decoding: same logits."""
    shape = synth.ModelShape(n_layers=2, d_model=128, n_heads=4, n_kv_heads=2, head_dim=64,
                             ffn_hidden=192, vocab=400, n_loops=3, window=8)
    weights = lively_weights(shape, 9, bf16=True, std=0.02)
    cfg = B.make_config(shape, dtype=B.PLT_BF16)
    model = B.Model(cfg, B.pack_weights(cfg, weights))
    prompts = synth.token_ids((2, 21), shape.vocab, 10)
    kv1 = B.KV(model, 2, 40)
    nxt, _ = kv1.prefill(dev_tokens(prompts))
    kv2 = B.KV(model, 2, 40)
    for seq in range(2):
        for layer in range(shape.n_layers):
            e = kv1.export(seq, layer, 21)
            assert e["k_share"].shape == (2, 21, 64) and e["k_ring"].shape == (2, 2, 8, 64)
            kv2.import_(seq, layer, 21, e["k_share"], e["v_share"], e["k_ring"], e["v_ring"])
    kv2.set_carry(kv1.get_carry())
    kv2.set_position(21)
    # exported keys equal the oracle's rotated keys (bf16-rounded) for one sequence
    orc = O.PLTOracle(oshape(shape), weights, kv_bf16=True)
    orc.clp_prefill(list(prompts[0]), 40)
    e = kv1.export(0, 1, 21)
    for got, ref in [(e["k_share"], orc.kv.ks[1, :21]), (e["v_share"], orc.kv.vs[1, :21]),
                     (e["k_ring"][0], orc.kv.kr[0, 1]), (e["v_ring"][1], orc.kv.vr[1, 1])]:
        err = float(np.max(np.abs(got - ref.transpose(1, 0, 2))))
        assert err <= 2e-2, err
    t = nxt.clone()
    a = kv1.decode_step(t)[1].cpu().numpy().copy()
    b = kv2.decode_step(t)[1].cpu().numpy().copy()
    assert np.array_equal(a, b)
    for k in (kv1, kv2):
        k.close()
    model.close()


def test_gemm_hook_matches_float64_product():
    rng = np.random.default_rng(0)
    for (M, N, K) in [(128, 192, 256), (37, 100, 64), (300, 70, 704), (8, 2048, 2048), (20, 70, 576),
                      (128, 1536, 2048), (192, 2048, 1152), (64, 1000, 2048), (256, 333, 640),
                      (512, 256, 128), (700, 390, 192), (1024, 1000, 64),
                      (160, 4096, 256), (150, 4100, 128), (192, 6144, 2048),    # 129..192 rows, wide: one 256 x 64 tile per 64 columns, three LDS stages
                      (300, 4096, 256), (1000, 4100, 128), (513, 6144, 512),     # 257.. rows, wide: several 256-row tiles (ragged last tile)
                      (4096, 4096, 128), (4100, 3100, 64)]:          # the last two take the 256 x 256 tile kernel
        a = synth.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
        w = synth.round_to_bf16(rng.standard_normal((N, K)).astype(np.float32))
        ref = a.astype(np.float64) @ w.astype(np.float64).T
        c = B.gemm(B.PLT_BF16, torch.from_numpy(a).cuda().to(torch.bfloat16), torch.from_numpy(w).cuda().to(torch.bfloat16))
        assert np.max(np.abs(c.cpu().numpy() - ref)) <= 1e-5 * K + 1e-4, (M, N, K)
        c32 = B.gemm(B.PLT_F32, torch.from_numpy(a).cuda(), torch.from_numpy(w).cuda())
        assert np.max(np.abs(c32.cpu().numpy() - ref)) <= 1e-5 * K + 1e-4, (M, N, K)


def test_gemm_residual_hook_adds_the_float64_product_in_place():
    """The prefill's output / down projections add their product to the residual stream in the tile kernel's epilogue:
    x += a w^T against the float64 product (ragged last row and column tiles included); other shapes are refused."""
    rng = np.random.default_rng(5)
    for (M, N, K) in [(4096, 4096, 128), (4100, 3101, 64), (16384, 1028, 192)]:
        a = synth.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
        w = synth.round_to_bf16(rng.standard_normal((N, K)).astype(np.float32))
        x0 = rng.standard_normal((M, N)).astype(np.float32) * 3
        ref = x0.astype(np.float64) + a.astype(np.float64) @ w.astype(np.float64).T
        x = torch.from_numpy(x0).cuda()
        B.gemm_residual(torch.from_numpy(a).cuda().to(torch.bfloat16), torch.from_numpy(w).cuda().to(torch.bfloat16), x)
        assert np.max(np.abs(x.cpu().numpy() - ref)) <= 1e-5 * K + 1e-4, (M, N, K)
    x = torch.zeros(128, 256, device="cuda")
    with pytest.raises(B.PltError):
        B.gemm_residual(torch.zeros(128, 64, device="cuda", dtype=torch.bfloat16), torch.zeros(256, 64, device="cuda", dtype=torch.bfloat16), x)
    assert float(x.abs().max()) == 0.0


@pytest.mark.parametrize("dtype,tol", [(B.PLT_F32, 2e-5), (B.PLT_BF16, 2e-2)])
def test_edge_cases_single_token_prompt_and_window_larger_than_context(dtype, tol):
    """Prompt of one token (position 0 sees only itself; every loop gets a zero shifted-in state),
    a window larger than the whole run, batch 1, and decoding right up to max_ctx."""
    shape = synth.ModelShape(n_layers=2, d_model=128, n_heads=4, n_kv_heads=2, head_dim=64,
                             ffn_hidden=192, vocab=300, n_loops=3, window=200)
    weights = lively_weights(shape, 21, bf16=dtype == B.PLT_BF16, std=0.02)
    prompts = synth.token_ids((1, 1), shape.vocab, 22)
    run_teacher_forced(shape, dtype, B.PLT_MODE_CLP, weights, prompts, 6, tol)


@pytest.mark.parametrize("mode", [B.PLT_MODE_CLP, B.PLT_MODE_CLP_SHARE_ONLY, B.PLT_MODE_CLP_OWN_KV, B.PLT_MODE_VANILLA_LOOP])
@pytest.mark.parametrize("kv_dtype", [0, B.PLT_FP8_E4M3], ids=["bf16kv", "e4m3kv"])
def test_decode_steps_of_more_than_128_rows_all_modes(mode, kv_dtype):
    """From 129 rows on the QKV projection of a decode step carries RoPE, the gate logit and the cache appends as its
    epilogue (64-row x 128-column tiles; row (b, l) at its sequence's own position): 48 sequences x 3 loops = 144 rows
    (three row tiles, the last ragged; 144 sequences in the sequential-loop mode), every mode's append rule, both cache
    types, against the oracle's teacher-forced steps."""
    shape = synth.ModelShape(n_layers=2, d_model=128, n_heads=4, n_kv_heads=2, head_dim=64,
                             ffn_hidden=192, vocab=300, n_loops=3, window=8)
    weights = lively_weights(shape, 51, bf16=True, std=0.02)
    Bn = 144 if mode == B.PLT_MODE_VANILLA_LOOP else 48
    n, steps = (9, 2) if mode == B.PLT_MODE_VANILLA_LOOP else (19, 3)
    prompts = synth.token_ids((Bn, n), shape.vocab, 52)
    run_teacher_forced(shape, B.PLT_BF16, mode, weights, prompts, steps, 4e-2 if kv_dtype else 2e-2, kv_dtype=kv_dtype)


@pytest.mark.parametrize("n_seq", [24, 48], ids=["72rows", "144rows"])
def test_decode_steps_with_a_wide_feed_forward_block(n_seq):
    """ffn_hidden = 12800 (200 tiles of 64 hidden columns): from 65 rows on the gate/up projection of a decode step
    takes tiles of 64 gate + 64 up columns (128 x 128 at up to 128 rows, 256 x 128 beyond), SwiGLU in the epilogue."""
    shape = synth.ModelShape(n_layers=1, d_model=128, n_heads=2, n_kv_heads=1, head_dim=64,
                             ffn_hidden=12800, vocab=300, n_loops=3, window=8)
    weights = lively_weights(shape, 61, bf16=True, std=0.02)
    prompts = synth.token_ids((n_seq, 9), shape.vocab, 62)
    run_teacher_forced(shape, B.PLT_BF16, B.PLT_MODE_CLP, weights, prompts, 2, 2e-2)


def test_window_one_and_many_loops():
    """w = 1: the window holds only the current position, so the local branch returns its own value row."""
    shape = synth.ModelShape(n_layers=1, d_model=64, n_heads=2, n_kv_heads=1, head_dim=64,
                             ffn_hidden=64, vocab=100, n_loops=6, window=1)
    weights = lively_weights(shape, 23, bf16=True, std=0.02)
    prompts = synth.token_ids((2, 7), shape.vocab, 24)
    run_teacher_forced(shape, B.PLT_BF16, B.PLT_MODE_CLP, weights, prompts, 5, 2e-2)


def test_prefill_then_prefill_restarts_the_cache():
    shape = synth.ModelShape(n_layers=1, d_model=64, n_heads=2, n_kv_heads=2, head_dim=64,
                             ffn_hidden=64, vocab=100, n_loops=2, window=4)
    weights = lively_weights(shape, 25, bf16=False, std=0.05)
    cfg = B.make_config(shape, dtype=B.PLT_F32)
    model = B.Model(cfg, B.pack_weights(cfg, weights))
    kv = B.KV(model, 1, 32)
    p1 = synth.token_ids((1, 20), shape.vocab, 26)
    p2 = synth.token_ids((1, 9), shape.vocab, 27)
    kv.prefill(dev_tokens(p1))
    a = kv.prefill(dev_tokens(p2))[1].cpu().numpy().copy()
    kv_fresh = B.KV(model, 1, 32)
    b = kv_fresh.prefill(dev_tokens(p2))[1].cpu().numpy().copy()
    assert kv.position == 9 and np.array_equal(a, b)
    # and the next decode step must not see anything of the first, longer prompt
    t = dev_tokens(np.array([5]))
    assert np.array_equal(kv.decode_step(t)[1].cpu().numpy(), kv_fresh.decode_step(t)[1].cpu().numpy())
    kv.close(); kv_fresh.close(); model.close()


@pytest.mark.parametrize("mode", [B.PLT_MODE_CLP_SHARE_ONLY, B.PLT_MODE_CLP_OWN_KV])
@pytest.mark.parametrize("dtype,tol", [(B.PLT_F32, 2e-5), (B.PLT_BF16, 2e-2)])
def test_ablation_modes(mode, dtype, tol):
    """Table 1 rows 3 and 4 in the same library: cross-loop parallel with per-loop KV, and with the
    shared first-loop KV but no window; kv bytes follow the table (L*n and n entries)."""
    shape = synth.ModelShape(n_layers=2, d_model=128, n_heads=4, n_kv_heads=2, head_dim=64,
                             ffn_hidden=192, vocab=400, n_loops=3, window=8)
    weights = lively_weights(shape, 41, bf16=dtype == B.PLT_BF16, std=0.02)
    prompts = synth.token_ids((2, 37), shape.vocab, 42)
    run_teacher_forced(shape, dtype, mode, weights, prompts, 7, tol)
    cfg = B.make_config(shape, dtype=dtype, mode=mode)
    model = B.Model(cfg, B.pack_weights(cfg, weights))
    es = 2 if dtype == B.PLT_BF16 else 4
    per = 2 * shape.n_layers * shape.n_kv_heads * shape.head_dim * es
    assert model.kv_logical_bytes(1, 1000) == per * 1000 * (3 if mode == B.PLT_MODE_CLP_OWN_KV else 1)
    model.close()
