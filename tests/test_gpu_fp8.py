"""e4m3 (FP8) K/V caches: parity of the HIP path (through the C ABI) with the CPU oracle.

Kernel level: the cache inputs are drawn already representable in e4m3, so both sides see exactly
the same numbers and the bf16 bars apply unchanged (2e-2 max-abs; 2^-8 * max|y| + 1e-3 from the
arithmetic: float statistics, bf16 softmax weights and outputs).

Model level: the device rounds K and V to e4m3 from float32 projections of bf16 activations, the
oracle from float64 ones.  An element whose two pre-rounding values straddle a rounding boundary
lands on neighbouring codes, one e4m3 step (2^-3 .. 2^-4 relative) apart, where the bf16 cache
would differ by 2^-8.  With pre-rounding differences of about 2^-9 relative that is expected for
roughly 2^-9 / 2^-4 = 3 % of the elements, and is checked as such: codes equal or adjacent, at most
6 % adjacent.  Logits are compared with the bar 4e-2 (twice the bf16 bar; see the design notes).
"""
import numpy as np
import pytest

from oracle import plt_oracle as O
from paper_2510_24824_amd import binding as B, synth
from tests.helpers import lively_weights, oshape
from tests.test_gpu_model import dev_tokens, run_teacher_forced

pytestmark = pytest.mark.gpu
FP8 = B.PLT_FP8_E4M3


def run_case(Bn, L, Hq, Hkv, D, N, w, seed, n_ctx=None, n_ring=None, splits=(0,), scale=1.0):
    a = synth.make_attn_inputs(Bn, L, Hq, Hkv, D, N, w, seed, bf16=True)
    for k in ("k_share", "v_share", "k_ring", "v_ring"):
        a[k] = synth.round_to_e4m3(a[k] * scale)
    ref = O.decode_attention(a["q"], a["k_share"], a["v_share"], a["k_ring"], a["v_ring"], a["z"],
                             n_ctx=n_ctx, n_ring=n_ring)
    dev = B.AttnDecode(FP8, a["q"], a["k_share"], a["v_share"], a["k_ring"], a["v_ring"], a["z"])
    outs = []
    for s in splits:
        y = dev.run(n_ctx=n_ctx, n_ring=n_ring, n_splits=s).float().cpu().numpy().astype(np.float64)
        err = np.max(np.abs(y - ref))
        assert err <= 2e-2 * scale, (s, err)
        assert err <= 2.0 ** -8 * np.max(np.abs(ref)) + 1e-3 * scale, (s, err, np.max(np.abs(ref)))
        outs.append(y)
    return outs, ref, dev


@pytest.mark.parametrize("case", [
    dict(Bn=3, L=3, Hq=16, Hkv=4, D=128, N=300, w=64),            # ragged N: 4 full tiles of 64 + 44 keys
    dict(Bn=2, L=2, Hq=4, Hkv=4, D=64, N=77, w=16),               # D = 64, window shorter than a tile
    dict(Bn=2, L=1, Hq=8, Hkv=2, D=128, N=130, w=1),              # non-looped: no ring at all
    dict(Bn=2, L=4, Hq=16, Hkv=2, D=64, N=200, w=40),             # L*G = 32 rows -> two row tiles
    dict(Bn=1, L=2, Hq=16, Hkv=16, D=128, N=1, w=64, n_ring=1),   # a single key
    dict(Bn=2, L=3, Hq=8, Hkv=4, D=128, N=1000, w=64, n_ctx=613, n_ring=29),  # partially filled caches
    dict(Bn=2, L=3, Hq=8, Hkv=2, D=128, N=500, w=150, n_ring=97),  # rings of several tiles, second one ragged
    dict(Bn=1, L=2, Hq=8, Hkv=8, D=128, N=64, w=64),              # exactly one full tile each
])
def test_fp8_attention_matches_oracle(case):
    run_case(seed=51, splits=(1, 2, 5, 0), **case)


def test_fp8_attention_large_and_tiny_values():
    """values near the top of the e4m3 range and down in its subnormals"""
    run_case(2, 3, 16, 4, 128, 500, 64, seed=52, splits=(1, 3), scale=60.0)
    a = synth.make_attn_inputs(2, 2, 8, 2, 128, 260, 64, 53, bf16=True)
    for k in ("v_share", "v_ring"):
        a[k] = synth.round_to_e4m3(a[k] * 2.0 ** -7)             # mostly subnormal codes
    for k in ("k_share", "k_ring"):
        a[k] = synth.round_to_e4m3(a[k])
    ref = O.decode_attention(a["q"], a["k_share"], a["v_share"], a["k_ring"], a["v_ring"], a["z"])
    y = B.AttnDecode(FP8, a["q"], a["k_share"], a["v_share"], a["k_ring"], a["v_ring"], a["z"]).run()
    assert np.max(np.abs(y.float().cpu().numpy() - ref)) <= 2.0 ** -8 * np.max(np.abs(ref)) + 1e-5


def test_fp8_attention_split_invariance_and_determinism():
    outs, ref, dev = run_case(4, 3, 16, 4, 128, 1500, 64, seed=54, splits=(1, 2, 3, 7, 16))
    for y in outs[1:]:
        assert np.max(np.abs(y - outs[0])) <= 2.0 ** -7 * np.max(np.abs(ref))
    again = [dev.run(n_splits=s).float().cpu().numpy() for s in (7, 7, 7)]
    assert np.array_equal(again[0], again[1]) and np.array_equal(again[1], again[2])


def test_fp8_attention_full_kernel_config():
    """Batch 32, L = 3, 16 query / 4 kv heads, D = 128, 4096 shared keys, window 64 -- every output."""
    outs, ref, dev = run_case(32, 3, 16, 4, 128, 4096, 64, seed=1, splits=(0,))
    assert ref.shape == (32, 3, 16, 128)


def test_fp8_every_code_reaches_the_matrix_cores_exactly():
    """V holds all 254 finite codes; a one-hot softmax (one huge score) returns each V row as is."""
    D, N = 128, 256
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], np.uint8)
    vals = synth.e4m3_from_bits(codes)                                   # 254 values
    v = np.zeros((1, 1, N, D), np.float32)
    v[0, 0, :, :] = vals[(np.arange(N)[:, None] * 7 + np.arange(D)[None, :]) % 254]
    k = np.zeros((1, 1, N, D), np.float32)
    q = np.zeros((1, 1, 1, D), np.float32)
    k[0, 0, :, 0] = 0.0; q[0, 0, 0, 0] = 256.0
    for target in (0, 63, 64, 130, 255):
        kk = k.copy(); kk[0, 0, target, 0] = 448.0                       # score 448*256/sqrt(128): one-hot
        y = B.AttnDecode(FP8, q, kk, v, np.zeros((1, 0, 1, 1, D), np.float32), np.zeros((1, 0, 1, 1, D), np.float32),
                         np.zeros((1, 0, 1), np.float32)).run().float().cpu().numpy()
        # bf16 output rounding of a value with <= 4 significant bits is exact
        assert np.array_equal(y[0, 0, 0], v[0, 0, target]), target


@pytest.mark.parametrize("L,w,heads,D", [(3, 8, (4, 2), 64), (2, 64, (2, 2), 128), (1, 1, (4, 4), 64), (4, 40, (8, 2), 64),
                                         (2, 100, (4, 4), 128)])
def test_fp8_small_models(L, w, heads, D):
    shape = synth.ModelShape(n_layers=2, d_model=128, n_heads=heads[0], n_kv_heads=heads[1], head_dim=D,
                             ffn_hidden=320, vocab=500, n_loops=L, window=w)
    weights = lively_weights(shape, 5, bf16=True, std=0.02)
    prompts = synth.token_ids((3, 45), shape.vocab, 6)
    run_teacher_forced(shape, B.PLT_BF16, B.PLT_MODE_CLP, weights, prompts, 12, 4e-2, kv_dtype=FP8)


@pytest.mark.parametrize("n,L,w,heads,D", [(333, 3, 40, (4, 2), 64), (200, 2, 100, (2, 2), 128)])
def test_fp8_prompts_of_several_key_tiles(n, L, w, heads, D):
    """As the bf16 test of the same name: prompts that span several 64-key steps and more than one 128-row query
    tile, lengths and windows that are no multiples of 32, with e4m3 caches."""
    shape = synth.ModelShape(n_layers=2, d_model=128, n_heads=heads[0], n_kv_heads=heads[1], head_dim=D,
                             ffn_hidden=320, vocab=500, n_loops=L, window=w)
    weights = lively_weights(shape, 9, bf16=True, std=0.02)
    prompts = synth.token_ids((2, n), shape.vocab, 12)
    run_teacher_forced(shape, B.PLT_BF16, B.PLT_MODE_CLP, weights, prompts, 4, 4e-2, kv_dtype=FP8)


@pytest.mark.parametrize("mode", [B.PLT_MODE_VANILLA_LOOP, B.PLT_MODE_CLP_SHARE_ONLY, B.PLT_MODE_CLP_OWN_KV])
def test_fp8_other_modes(mode):
    shape = synth.ModelShape(n_layers=2, d_model=128, n_heads=4, n_kv_heads=2, head_dim=64,
                             ffn_hidden=192, vocab=400, n_loops=3, window=8)
    weights = lively_weights(shape, 41, bf16=True, std=0.02)
    prompts = synth.token_ids((2, 37), shape.vocab, 42)
    run_teacher_forced(shape, B.PLT_BF16, mode, weights, prompts, 7, 4e-2, kv_dtype=FP8)


def test_fp8_cache_codes_and_bytes():
    """The exported cache holds the oracle's e4m3 codes, up to neighbouring codes where the two sides'
    pre-rounding values straddle a boundary; export / import round-trips bit-exactly; the cache is
    half the bf16 one."""
    shape = synth.ModelShape(n_layers=2, d_model=128, n_heads=4, n_kv_heads=2, head_dim=64,
                             ffn_hidden=192, vocab=400, n_loops=3, window=8)
    weights = lively_weights(shape, 9, bf16=True, std=0.02)
    cfg = B.make_config(shape, dtype=B.PLT_BF16, kv_dtype=FP8)
    model = B.Model(cfg, B.pack_weights(cfg, weights))
    cfg16 = B.make_config(shape, dtype=B.PLT_BF16)
    model16 = B.Model(cfg16, B.pack_weights(cfg16, weights))
    assert 2 * model.kv_logical_bytes(3, 1000) == model16.kv_logical_bytes(3, 1000)
    assert model.kv_logical_bytes(1, 1000) == O.kv_cache_bytes(oshape(shape), 1000, 1)
    prompts = synth.token_ids((2, 21), shape.vocab, 10)
    kv1 = B.KV(model, 2, 40)
    nxt, _ = kv1.prefill(dev_tokens(prompts))
    orc = O.PLTOracle(oshape(shape), weights, kv_fp8=True)
    orc.clp_prefill(list(prompts[0]), 40)
    total = adjacent = 0
    for layer in (0, 1):
        e = kv1.export(0, layer, 21)
        for i, (got, ref) in enumerate([(e["k_share"], orc.kv.ks[layer, :21]), (e["v_share"], orc.kv.vs[layer, :21]),
                                        (e["k_ring"][0], orc.kv.kr[0, layer]), (e["v_ring"][1], orc.kv.vr[1, layer])]):
            ref = ref.transpose(1, 0, 2).astype(np.float32)
            assert np.array_equal(synth.round_to_e4m3(got), got)         # every stored byte is a finite code
            # pre-rounding values within the bf16 bar of each other, each rounded by at most half a step
            # (a step is at most 2^-3 of the value):
            excess = float(np.max(np.abs(got - ref) - 2.0 ** -3 * np.maximum(np.abs(got), np.abs(ref))))
            assert excess <= 2e-2, excess
            if layer == 0 and i < 2:
                # first layer, first loop: the pre-rounding values differ only by the rounding of the
                # projection's inputs, so normal-range elements land on the same or on neighbouring codes
                nrm = np.abs(ref) >= 2.0 ** -6
                cg, cr = synth.e4m3_bits(got).astype(np.int32), synth.e4m3_bits(ref).astype(np.int32)
                diff = np.abs((cg & 0x7F) * np.where(cg & 0x80, -1, 1) - (cr & 0x7F) * np.where(cr & 0x80, -1, 1))[nrm]
                assert int(diff.max()) <= 1, int(diff.max())
                total += diff.size; adjacent += int((diff == 1).sum())
    print(f"first layer, first loop, normal range: {adjacent} of {total} elements on a neighbouring code")
    assert adjacent <= 0.06 * total
    kv2 = B.KV(model, 2, 40)
    for seq in range(2):
        for layer in range(shape.n_layers):
            ex = kv1.export(seq, layer, 21)
            kv2.import_(seq, layer, 21, ex["k_share"], ex["v_share"], ex["k_ring"], ex["v_ring"])
            back = kv2.export(seq, layer, 21)
            assert all(np.array_equal(ex[k], back[k]) for k in ex)
    kv2.set_carry(kv1.get_carry()); kv2.set_position(21)
    t = nxt.clone()
    assert np.array_equal(kv1.decode_step(t)[1].cpu().numpy(), kv2.decode_step(t)[1].cpu().numpy())
    for k in (kv1, kv2):
        k.close()
    model.close(); model16.close()


def test_fp8_needs_bf16_model():
    shape = synth.TINY
    cfg = B.make_config(shape, dtype=B.PLT_F32, kv_dtype=FP8)
    with pytest.raises(B.PltError):
        B.pack_weights(cfg, synth.make_weights(shape, 0, bf16=False))
