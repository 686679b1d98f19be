"""Low-bit (microscaling) projections: the device quantisers and the block-scaled GEMM against the oracle.

The quantisers decide integers (codes, scale bytes) from floats; both sides get the same float32 / bf16
inputs, and every step of the rule (power-of-two scaling, rounding to the element grid) is exact in float,
so codes and scales must be bit-identical.  The GEMM multiplies the codes exactly (products of grid values)
and accumulates in float: it is compared with the float64 product of the dequantised operands within an
element-wise bound from the accumulation alone."""
import numpy as np
import pytest
import torch

from oracle import plt_oracle as O
from paper_2510_24824_amd import binding as B, synth
from tests.helpers import lively_weights
from tests.test_gpu_model import run_teacher_forced

pytestmark = pytest.mark.gpu


def decode_weights(codes, scales, N, K):
    """Device layout -> (element values [N, K], exponents [N, K/32]) using the layout's closed form."""
    codes, scales = codes.cpu().numpy(), scales.cpu().numpy()
    n = np.arange(N)[:, None]; k = np.arange(K)[None, :]
    byte = ((n >> 4) * (K >> 7) + (k >> 7)) * 1024 + (((k >> 5) & 3) * 16 + (n & 15)) * 16 + ((k & 31) >> 1)
    nib = np.where(k & 1, codes[byte] >> 4, codes[byte] & 15)
    b = np.arange(K // 32)[None, :]
    n_cgrp = ((K >> 7) + 3) >> 2
    sidx = (((n >> 4) * n_cgrp + (b >> 4)) * 64 + (b & 3) * 16 + (n & 15)) * 4 + ((b >> 2) & 3)
    return synth.e2m1_from_bits(nib).astype(np.float64), scales[sidx].astype(np.int64) - 127


def decode_acts(codes, scales, M, K):
    codes, scales = codes.cpu().numpy(), scales.cpu().numpy()
    b = np.arange(K // 32)
    sidx = (b >> 4) * 16 + (b & 3) * 4 + ((b >> 2) & 3)
    return synth.e4m3_from_bits(codes).astype(np.float64), scales[:, sidx].astype(np.int64) - 127


def test_layout_closed_forms_match_the_abi():
    l = B.lib()
    K = 640
    for n, k in [(0, 0), (17, 33), (31, 639), (5, 128), (40, 511)]:
        want = ((n >> 4) * (K >> 7) + (k >> 7)) * 1024 + (((k >> 5) & 3) * 16 + (n & 15)) * 16 + ((k & 31) >> 1)
        assert l.plt_mx_weight_code_index(n, k, K) == want
        b = k >> 5
        assert l.plt_mx_weight_scale_index(n, b, K) == (((n >> 4) * 2 + (b >> 4)) * 64 + (b & 3) * 16 + (n & 15)) * 4 + ((b >> 2) & 3)
    assert [l.plt_mx_act_scale_index(b) for b in (0, 1, 4, 5, 15, 16, 21)] == [0, 4, 1, 5, 15, 16, 16 + 4 + 1]
    assert l.plt_mx_weight_code_bytes(48, 640) == 48 * 320 and l.plt_mx_weight_scale_bytes(48, 640) == 3 * 2 * 256
    assert l.plt_mx_act_scale_bytes(7, 640) == 7 * 32
    assert l.plt_mx_weight_code_bytes(40, 640) == 0 and l.plt_mx_weight_code_bytes(48, 600) == 0


def _weights(N, K, seed):
    w = synth.normal((N, K), seed, 70, 0.02, True)
    w[0, :32] = 0.0                                         # an all-zero block
    w[1, :64] *= 2.0 ** 40; w[2, :64] *= 2.0 ** -60         # large and tiny blocks
    # exact ties of the e2m1 grid at block scale 1 (maximum 6 -> exponent 0): 0.25 .75 1.25 1.75 2.5 3.5 5
    w[3, :32] = 0.0; w[3, :9] = [6.0, 0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, -2.5]
    w[4, :32] = 0.0; w[4, :3] = [7.5, -7.0, 0.3]            # 7.5 and 7 exceed the largest element: saturate to 6
    return synth.round_to_bf16(w)


@pytest.mark.parametrize("N,K", [(48, 640), (6144, 2048), (16, 128)])
def test_weight_quantiser_is_bit_exact(N, K):
    w = _weights(N, K, 5)
    codes, scales = B.mx_quantize_weights(torch.from_numpy(w).cuda().to(torch.bfloat16))
    got_q, got_e = decode_weights(codes, scales, N, K)
    want_q, want_e = O.mx_quantize(w, "e2m1")
    assert np.array_equal(got_e, want_e)
    assert np.array_equal(got_q, want_q)
    assert list(got_q[3, :9]) == [6.0, 0.0, 1.0, 1.0, 2.0, 2.0, 4.0, 4.0, -2.0] and list(got_q[4, :2]) == [6.0, -6.0]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("M,K", [(37, 640), (128, 2048), (3, 32)])
def test_activation_quantiser_is_bit_exact(dtype, M, K):
    x = synth.normal((M, K), 6, 71, 1.0, dtype == torch.bfloat16)
    x[0, :32] = 0.0
    x[1 % M, :32] *= 1e-30
    x[2 % M, 0] = 500.0; x[2 % M, 1] = 465.0                 # block maximum 500: exponent 0; 500 and 465 saturate to 448
    if dtype == torch.bfloat16:
        x = synth.round_to_bf16(x)
    codes, scales = B.mx_quantize_act(torch.from_numpy(x).cuda().to(dtype))
    got_q, got_e = decode_acts(codes, scales, M, K)
    want_q, want_e = O.mx_quantize(x, "e4m3")
    assert np.array_equal(got_e, want_e)
    assert np.array_equal(got_q, want_q)
    assert got_q[2 % M, 0] == 448.0 and got_q[2 % M, 1] == 448.0
    pad = np.setdiff1d(np.arange(scales.shape[1]), [(b >> 4) * 16 + (b & 3) * 4 + ((b >> 2) & 3) for b in range(K // 32)])
    assert np.all(scales.cpu().numpy()[:, pad] == 0)         # scale bytes of blocks beyond K


GEMM_CASES = [(128, 6144, 2048),   # QKV projection of the 1.3B model at 64 sequences x 2 loops
              (128, 2048, 5632),   # down projection: 5.5 K ranges (a ragged last range)
              (64, 2048, 2048),    # output projection, 64 rows (two workgroups per compute unit)
              (256, 11264, 2048),  # gate/up at L = 4: two row blocks, four strips per wave task
              (37, 80, 384),       # nothing a multiple of a tile
              (130, 2048, 1024),   # second row block with two rows
              (1, 16, 128),
              (2048, 4096, 640),   # prefill-sized: the 256 x 256-tile kernel, whole K (5 chunks: a partial scale group)
              (1100, 6640, 256),   # the tiled kernel with ragged last row and column tiles
              (200, 2048, 640),    # row tiles: four 64-row tiles, the last with a ragged tail, 5 chunks (a partial scale group)
              (384, 1040, 1536),   # row tiles: six row tiles, a ragged last column tile, three K runs
              (16, 256, 512)]      # row tiles: the smallest shape they take (one scale group, four column tiles)


@pytest.mark.parametrize("M,N,K", GEMM_CASES)
def test_gemm_mx_matches_oracle(M, N, K):
    w = synth.normal((N, K), 7, 72, 0.02, True)
    x = synth.normal((M, K), 7, 73, 1.0, False)
    x[:, : K // 2] *= np.exp(synth.normal((M, 1), 7, 74, 2.0, False))       # rows and halves on different scales
    wc, ws = B.mx_quantize_weights(torch.from_numpy(w).cuda().to(torch.bfloat16))
    ac, asc = B.mx_quantize_act(torch.from_numpy(x).cuda())
    got = B.gemm_mx(ac, asc, wc, ws, M, N, K).cpu().numpy()
    wq, we = O.mx_quantize(w, "e2m1")
    aq, ae = O.mx_quantize(x, "e4m3")
    wd, ad = O.mx_dequantize(wq, we), O.mx_dequantize(aq, ae)
    ref = ad @ wd.T
    # products are exact; the instruction adds the 128 products of a step after aligning them to a common
    # exponent (a fixed-point sum narrower than a chain of float additions: measured up to 2^-17.9 of the sum
    # of |terms|, independent of K), then the float accumulator and the slab additions round as usual
    bound = 2.0 ** -16 * (np.abs(ad) @ np.abs(wd).T) + 1e-30
    err = np.abs(got - ref)
    print(f"max |c| {np.abs(ref).max():.3e}; max err {err.max():.3e}; max err / bound {np.max(err / bound):.3f}")
    assert np.all(err <= bound)
    # and the quantised product is close to the unquantised one (sanity of the whole chain)
    exact = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.abs(ref - exact).max() <= 0.25 * np.abs(exact).max()


SWIGLU_CASES = [(128, 5632, 2048),   # gate/up of the 1.3B model at 64 sequences x 2 loops: one kernel, SwiGLU + quantiser in its epilogue
                (64, 4096, 512),     # one scale group
                (200, 4096, 640),    # four row tiles, the last with a ragged tail, a partial scale group
                (300, 4128, 1024),   # five row tiles, F / 32 = 129 column tiles
                (1, 4096, 512),
                (40, 1024, 384)]     # too narrow for the fused kernel: product slabs + the activation kernel


@pytest.mark.parametrize("M,F,K", SWIGLU_CASES)
def test_gemm_mx_swiglu_matches_oracle(M, F, K):
    """h = silu(a Wg^T) * (a Wu^T) quantised to e4m3 blocks by the device against the oracle's float64 evaluation of
    the same chain from the same quantised operands.  The quantiser decides integers from floats that differ in
    their last bits (float32 accumulation on the device), so: the scale byte of a block equals the oracle's unless
    the block maximum lies within float accumulation error of a power of two; with the same scale every code is
    the oracle's or its neighbour on the e4m3 grid (plus the accumulation error for elements far below the row's
    largest); at most 2 % of the codes differ, and without bias (a wrong
    activation formula, operand order, gate/up swap or block assignment fails all of these at once)."""
    w = synth.normal((2 * F, K), 11, 82, 0.05, True)
    x = synth.normal((M, K), 11, 83, 1.0, False)
    x[:, : K // 2] *= np.exp(synth.normal((M, 1), 11, 84, 1.0, False))
    wc, ws = B.mx_quantize_weights(torch.from_numpy(w).cuda().to(torch.bfloat16))
    ac, asc = B.mx_quantize_act(torch.from_numpy(x).cuda())
    hc, hs = B.gemm_mx_swiglu(ac, asc, wc, ws, M, F, K)
    dev_q, dev_e = decode_acts(hc, hs, M, F)
    pad = np.setdiff1d(np.arange(hs.shape[1]), [(b >> 4) * 16 + (b & 3) * 4 + ((b >> 2) & 3) for b in range(F // 32)])
    assert np.all(hs.cpu().numpy()[:, pad] == 0)
    wq, we = O.mx_quantize(w, "e2m1")
    aq, ae = O.mx_quantize(x, "e4m3")
    gu = O.mx_dequantize(aq, ae) @ O.mx_dequantize(wq, we).T
    g, u = gu[:, :F], gu[:, F:]
    h = g / (1.0 + np.exp(-g)) * u
    own_q, own_e = O.mx_quantize(h, "e4m3")
    own = O.mx_dequantize(own_q, own_e)
    dev = dev_q * np.repeat(np.ldexp(1.0, dev_e), 32, axis=1)
    same = own_e == dev_e
    amax = np.abs(h).reshape(M, F // 32, 32).max(axis=2)
    mant = amax / np.exp2(np.floor(np.log2(np.maximum(amax, 1e-300))))                          # in [1, 2)
    near_pow2 = np.minimum(mant - 1.0, 2.0 - mant) <= 1e-4                                      # block maximum next to a power of two
    assert np.all(same | near_pow2), np.argwhere(~(same | near_pow2))[:8]
    s32 = np.repeat(same, 32, axis=1)
    mag = np.maximum(np.abs(own), np.abs(dev)) / np.repeat(np.ldexp(1.0, own_e), 32, axis=1)
    step = np.ldexp(1.0, np.maximum(np.floor(np.log2(np.maximum(mag, 2.0 ** -20))), -6).astype(np.int64) - 3) * np.repeat(np.ldexp(1.0, own_e), 32, axis=1)
    # the products carry the float accumulation error of 2048 terms (an ABSOLUTE error, 2^-16 of the sum of |terms|):
    # elements far below their row's largest may move by more than one of their own (finer) steps
    slack = 2.0 ** -12 * np.max(np.abs(h), axis=1, keepdims=True)
    ok = np.where(s32, np.abs(dev - own) <= step * (1 + 1e-9) + slack, np.abs(dev - h) <= 2.0 ** -3 * np.abs(h) + step + slack)
    assert np.all(ok), (np.argwhere(~ok)[:8], dev[~ok][:8], own[~ok][:8])
    n_diff = int(np.sum(dev != own))
    big = np.abs(own) > 0.05 * np.max(np.abs(own), axis=1, keepdims=True)
    bias = abs(float(np.mean((dev[big] - own[big]) / own[big])))
    print(f"codes that are the oracle's neighbour: {n_diff} of {dev.size}; blocks with another scale byte: {int(np.sum(~same))}; "
          f"mean signed deviation {bias:.2e}")
    assert n_diff <= 0.02 * dev.size and bias <= 2e-3


def test_gemm_mx_rejects_bad_shapes():
    z = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    for M, N, K in [(4, 40, 128), (4, 48, 96), (0, 48, 128)]:
        c = torch.zeros(max(M, 1), N, device="cuda")
        assert B.lib().plt_gemm_mx(M, N, K, B._ptr(z), B._ptr(z), B._ptr(z), B._ptr(z), B._ptr(c), B._ptr(z), z.numel(), None) == -1


MX_SMALL = synth.ModelShape(n_layers=2, d_model=128, n_heads=2, n_kv_heads=1, head_dim=64, ffn_hidden=256,
                            vocab=300, n_loops=3, window=5)


@pytest.mark.parametrize("mode,kv_dtype", [(B.PLT_MODE_CLP, 0), (B.PLT_MODE_VANILLA_LOOP, 0), (B.PLT_MODE_CLP, B.PLT_FP8_E4M3)])
def test_model_with_lowbit_projections(mode, kv_dtype):
    """Whole model with the four per-layer projections on MXFP4 weights / MXFP8 activations against the oracle's
    w_mx model (same quantisation rule, float64 arithmetic)."""
    weights = lively_weights(MX_SMALL, 9, bf16=True, std=0.05)
    prompts = synth.token_ids((2, 9), MX_SMALL.vocab, 10)
    run_teacher_forced(MX_SMALL, B.PLT_BF16, mode, weights, prompts, 6, MX_MODEL_TOL, kv_dtype=kv_dtype, w_dtype=B.PLT_MXFP4)


@pytest.mark.parametrize("mode", [B.PLT_MODE_CLP, B.PLT_MODE_CLP_SHARE_ONLY, B.PLT_MODE_CLP_OWN_KV, B.PLT_MODE_VANILLA_LOOP])
@pytest.mark.parametrize("kv_dtype", [0, B.PLT_FP8_E4M3], ids=["bf16kv", "e4m3kv"])
def test_lowbit_decode_steps_of_more_than_64_rows_all_modes(mode, kv_dtype):
    """From 65 rows on the low-bit QKV projection of a decode step carries RoPE, the gate logit and the cache appends as
    its epilogue (64-row x 128-column tiles, two heads of 64 per wave; row (b, l) at its sequence's own position):
    24 sequences x 3 loops = 72 rows (two row tiles, the second ragged; 72 sequences in the sequential-loop mode),
    every mode's append rule, both cache types.  Free-running low-bit bar, 8 % of the state's magnitude (4.2 with
    these prompts; measured up to 0.25 with e4m3 caches over 24 sequences); a wrong ring slot, cache or position is off
    by the state's full size."""
    weights = lively_weights(MX_SMALL, 9, bf16=True, std=0.05)
    Bn = 72 if mode == B.PLT_MODE_VANILLA_LOOP else 24
    n, steps = (6, 2) if mode == B.PLT_MODE_VANILLA_LOOP else (9, 3)
    prompts = synth.token_ids((Bn, n), MX_SMALL.vocab, 53)
    run_teacher_forced(MX_SMALL, B.PLT_BF16, mode, weights, prompts, steps, 0.08 * 4.2, kv_dtype=kv_dtype, w_dtype=B.PLT_MXFP4)


@pytest.mark.parametrize("kv_dtype", [0, B.PLT_FP8_E4M3], ids=["bf16kv", "e4m3kv"])
def test_lowbit_decode_steps_of_more_than_64_rows_heads_of_128(kv_dtype):
    """The same epilogue with heads of 128 (one head per wave), 512 hidden rows per head group so that the attention
    kernel also writes its output as e4m3 blocks: 22 sequences x 3 loops = 66 rows."""
    shape = synth.ModelShape(n_layers=2, d_model=256, n_heads=4, n_kv_heads=2, head_dim=128, ffn_hidden=256,
                             vocab=300, n_loops=3, window=5)
    weights = lively_weights(shape, 13, bf16=True, std=0.05)
    prompts = synth.token_ids((22, 7), shape.vocab, 54)
    run_teacher_forced(shape, B.PLT_BF16, B.PLT_MODE_CLP, weights, prompts, 3, 0.08 * 9.0, kv_dtype=kv_dtype, w_dtype=B.PLT_MXFP4)


def test_lowbit_model_single_position():
    """One position, L = 1: softmax over a single key returns the (bf16-stored) value row on both sides, so the
    values entering a quantiser differ only by float-level arithmetic -- dominated by the matrix-core
    instruction's fixed-point block sums, about 1e-4 relative.  A quantiser turns such a difference into a
    changed e4m3 code (one grid step, 6-12 % of that element) for about 1e-4 / 2^-4 = 0.2 % of the elements:
    a fraction of a flip per row and projection, each worth about 1 / sqrt(K) * 10 % of that projection's
    output.  Bar: 3 % of the largest logit (1.84; measured 1.8 %); a wrong layout, scale tensor or operand order
    is off by 100 %."""
    from tests.helpers import with_shape
    shape = with_shape(MX_SMALL, n_loops=1)
    weights = lively_weights(shape, 11, bf16=True, std=0.05)
    prompts = synth.token_ids((8, 1), shape.vocab, 12)
    run_teacher_forced(shape, B.PLT_BF16, B.PLT_MODE_CLP, weights, prompts, 0, 0.03 * 1.84, w_dtype=B.PLT_MXFP4)


# Several positions and loops: bf16 queries, softmax weights and attention outputs move the quantiser inputs by
# about 2^-9, so about 2^-9 / 2^-4 = 3 % of the e4m3 codes differ by one step between the two sides; a projection
# output then differs by about sqrt(0.03) * 2^-4.5 = 0.8 % (rms), and the differences add up over 4 projections,
# 2 layers and the loop-to-loop carry: a few per cent of the state's magnitude (~3), measured 0.13-0.15 max-abs;
# the bar is 8 % of that magnitude.
MX_MODEL_TOL = 0.25


MX_MOE = synth.ModelShape(n_layers=2, d_model=128, n_heads=2, n_kv_heads=2, head_dim=64, ffn_hidden=128, vocab=300,
                          n_loops=2, window=5, n_experts=6, top_k=2)


def test_moe_model_with_lowbit_experts_single_position():
    """Mixture of experts on low-bit operands, one position and L = 1 (no code flips from attention, see the dense
    single-position test): router on the quantised row, grouped block-scaled GEMMs, hidden rows quantised in the
    gate/up epilogue.  Seed chosen (from the oracle alone) so that every routing gap exceeds 0.05."""
    from tests.helpers import with_shape
    from tests.helpers import oshape
    shape = with_shape(MX_MOE, n_loops=1)
    weights = lively_weights(shape, MX_MOE_SEED, bf16=True, std=0.05, router_std=0.2)
    prompts = synth.token_ids((8, 1), shape.vocab, MX_MOE_SEED + 1)
    gaps = []
    for b in range(8):
        orc = O.PLTOracle(oshape(shape), weights, kv_bf16=True, w_mx=True)
        orc.greedy_generate(list(prompts[b]), 0)
        gaps += orc.route_margins
    assert min(gaps) > 0.05, min(gaps)
    run_teacher_forced(shape, B.PLT_BF16, B.PLT_MODE_CLP, weights, prompts, 0, 2e-2, w_dtype=B.PLT_MXFP4)


@pytest.mark.parametrize("mode,kv_dtype,seed", [(B.PLT_MODE_CLP, 0, 8), (B.PLT_MODE_CLP, B.PLT_FP8_E4M3, 8),
                                                 (B.PLT_MODE_VANILLA_LOOP, 0, 8)])
def test_moe_model_with_lowbit_experts(mode, kv_dtype, seed):
    """Several positions and loops; tolerance and its reason as for the dense low-bit model above.  Routing gaps
    of the oracle (router logits are ~N(0, 2.3)) are printed; a gap below the logit noise that flipped e4m3
    codes cause may route a row differently on the two sides, which the bar (8 % of the state's size) absorbs
    for near-tied experts only."""
    from tests.helpers import oshape
    fp8 = kv_dtype == B.PLT_FP8_E4M3
    weights = lively_weights(MX_MOE, seed, bf16=True, std=0.05, router_std=0.2)
    prompts = synth.token_ids((2, 4), MX_MOE.vocab, seed + 2)
    if mode == B.PLT_MODE_CLP:
        gaps = []
        for b in range(2):
            orc = O.PLTOracle(oshape(MX_MOE), weights, kv_bf16=not fp8, kv_fp8=fp8, w_mx=True)
            orc.greedy_generate(list(prompts[b]), 3)
            gaps += orc.route_margins
        print(f"smallest routing gap of the oracle: {min(gaps):.4f}")
        if not fp8:
            assert min(gaps) > 0.05, min(gaps)
    run_teacher_forced(MX_MOE, B.PLT_BF16, mode, weights, prompts, 3, MX_MODEL_TOL, kv_dtype=kv_dtype, w_dtype=B.PLT_MXFP4)


MX_MOE_SEED = 0


@pytest.mark.parametrize("rows,E,k", [(40, 4, 2), (70, 4, 2), (150, 4, 2), (1100, 4, 2), (2100, 4, 2)])
def test_moe_lowbit_tile_variants_single_position(rows, E, k):
    """20, 35 and 75 rows per expert on average: the 32-row, 64-row and 128-row tiles of the grouped low-bit
    GEMM (several tiles per expert); 550 rows per expert: the prefill-sized 256 x 256-tile kernel (sorted lists, ragged
    row tiles); 2100 rows: the router's prefill-sized launch on e4m3 rows; on single-position L = 1 sequences where the
    comparison is tight."""
    from tests.helpers import oshape, with_shape
    shape = with_shape(MX_MOE, n_loops=1, n_experts=E, top_k=k, n_layers=1)
    weights = lively_weights(shape, 3, bf16=True, std=0.05, router_std=0.2)
    prompts = synth.token_ids((rows, 1), shape.vocab, 4)
    run_teacher_forced(shape, B.PLT_BF16, B.PLT_MODE_CLP, weights, prompts, 0, 2e-2, w_dtype=B.PLT_MXFP4)


def test_moe_lowbit_full_width_single_position():
    """The 8-of-64 recipe's matrix widths (hidden 2048 = two K ranges of the grouped kernel, 16 heads of 128,
    experts of hidden 1024) with 8 experts, 2 per row, two layers; 64 single-position L = 1 sequences, so that
    the comparison with the oracle stays tight (see the single-position tests above).  The second layer's router
    sees a row that already carries a few flipped e4m3 codes (about 1 % of its logits' spread), so a sequence is
    compared only if the oracle's routing gaps all exceed 0.1 (logits ~N(0, 1.6)); most must qualify."""
    from tests.helpers import oshape
    from tests.test_gpu_model import dev_tokens
    shape = synth.ModelShape(n_layers=2, d_model=2048, n_heads=16, n_kv_heads=16, head_dim=128, ffn_hidden=1024,
                             vocab=2000, n_loops=1, window=64, n_experts=8, top_k=2)
    weights = lively_weights(shape, 21, bf16=True, std=0.02, router_std=0.05)
    prompts = synth.token_ids((64, 1), shape.vocab, 22)
    cfg = B.make_config(shape, dtype=B.PLT_BF16, w_dtype=B.PLT_MXFP4)
    model = B.Model(cfg, B.pack_weights(cfg, weights))
    kv = B.KV(model, 64, 4)
    _, lg = kv.prefill(dev_tokens(prompts))
    got = lg.cpu().numpy()
    orc = O.PLTOracle(oshape(shape), weights, kv_bf16=True, w_mx=True)
    compared, worst, top, rel_rms = 0, 0.0, 0.0, []
    for b in range(64):
        orc.route_margins = []
        _, ref = orc.clp_prefill(list(prompts[b]), 4)
        if min(orc.route_margins) <= 0.1:
            continue
        compared += 1
        worst = max(worst, float(np.max(np.abs(got[b] - ref)))); top = max(top, float(np.max(np.abs(ref))))
        rel_rms.append(float(np.sqrt(np.mean((got[b] - ref) ** 2) / np.mean(ref ** 2))))
    print(f"compared {compared} of 64 sequences; worst abs err {worst:.3e}; max |logit| {top:.3f}; "
          f"relative rms error median {np.median(rel_rms):.3e} max {np.max(rel_rms):.3e}")
    # 2048-wide rows: each quantiser sees a handful of flipped codes per row (0.2 % of 2048), so no sequence is
    # exact; most agree to the bf16 level of the head (measured median relative rms 0.6 %), the worst to 3 %
    assert compared >= 40 and np.median(rel_rms) <= 1.5e-2 and worst <= 0.05 * top
    kv.close(); model.close()


def test_lowbit_prefill_sized_gate_up_projection_single_position():
    """2048 rows through a layer with a 2048-wide SwiGLU: the gate/up projection (2048 x 4096 x 256) is large enough
    for the 256 x 256-tile low-bit kernel inside the model (whole K, one float slab; the other projections of this
    shape stay on the streaming kernel), followed by the SwiGLU + quantiser kernel.  2048 single-position L = 1
    sequences, compared as in the full-width MoE test: most sequences to the bf16 level of the head, the worst
    within 5 % of the largest logit."""
    from tests.helpers import oshape
    from tests.test_gpu_model import dev_tokens
    shape = synth.ModelShape(n_layers=1, d_model=256, n_heads=2, n_kv_heads=2, head_dim=128, ffn_hidden=2048,
                             vocab=300, n_loops=1, window=8)
    weights = lively_weights(shape, 31, bf16=True, std=0.05)
    n_seq = 2048
    prompts = synth.token_ids((n_seq, 1), shape.vocab, 32)
    cfg = B.make_config(shape, dtype=B.PLT_BF16, w_dtype=B.PLT_MXFP4)
    model = B.Model(cfg, B.pack_weights(cfg, weights))
    kv = B.KV(model, n_seq, 4)
    _, lg = kv.prefill(dev_tokens(prompts))
    got = lg.cpu().numpy()
    orc = O.PLTOracle(oshape(shape), weights, kv_bf16=True, w_mx=True)
    refs = {}
    for b in range(n_seq):                               # 300 distinct tokens: one oracle run per token
        t = int(prompts[b, 0])
        if t not in refs:
            refs[t] = orc.clp_prefill([t], 4)[1]
    ref = np.stack([refs[int(prompts[b, 0])] for b in range(n_seq)])
    top = float(np.max(np.abs(ref)))
    worst = float(np.max(np.abs(got - ref)))
    rel_rms = np.sqrt(np.mean((got - ref) ** 2, axis=1) / np.mean(ref ** 2, axis=1))
    print(f"{len(refs)} distinct tokens; worst abs err {worst:.3e}; max |logit| {top:.3f}; relative rms error median "
          f"{np.median(rel_rms):.3e} max {np.max(rel_rms):.3e}")
    assert np.median(rel_rms) <= 1.5e-2 and worst <= 0.05 * top
    kv.close(); model.close()


@pytest.mark.parametrize("heads,D,kv_dtype", [((4, 2), 128, 0), ((8, 8), 64, B.PLT_FP8_E4M3)])
def test_lowbit_model_with_attention_output_quantised_in_the_kernel(heads, D, kv_dtype):
    """n_heads * head_dim = 512: in decode steps the attention kernel itself writes its output as e4m3 blocks
    (no bf16 rounding, no quantiser launch).  Same statistical bar as the other multi-position low-bit tests,
    8 % of the state's magnitude (9.0 here; measured 0.42-0.54, and the same with a separate quantiser kernel); a
    wrong block, scale byte or row would be off by the state's full size."""
    shape = synth.ModelShape(n_layers=2, d_model=256, n_heads=heads[0], n_kv_heads=heads[1], head_dim=D,
                             ffn_hidden=256, vocab=300, n_loops=3, window=5)
    weights = lively_weights(shape, 13, bf16=True, std=0.05)
    prompts = synth.token_ids((3, 7), shape.vocab, 14)
    run_teacher_forced(shape, B.PLT_BF16, B.PLT_MODE_CLP, weights, prompts, 6, 0.08 * 9.0, kv_dtype=kv_dtype, w_dtype=B.PLT_MXFP4)


MX_WIDE = synth.ModelShape(n_layers=2, d_model=512, n_heads=4, n_kv_heads=2, head_dim=128, ffn_hidden=4096,
                           vocab=300, n_loops=3, window=5)


@pytest.mark.parametrize("shape", [MX_SMALL, MX_WIDE], ids=["small", "wide-ffn"])
def test_lowbit_layers_from_the_devices_own_activation_codes(shape):
    """A low-bit layer compared WITHOUT the rounding-boundary ambiguity of the quantisers.  A quantiser decides an
    integer from a float; device (float32, bf16 attention internals) and oracle (float64) inputs differ in the last
    bits, so a few per cent of the codes legitimately differ by one step and a free-running comparison needs a wide
    bar (MX_MODEL_TOL).  Here every layer of the device gets the oracle's layer input (plt_debug_layer), the e4m3 codes
    and scales that entered its four projections are read back (plt_debug_act_codes), and the oracle evaluates the
    same layer with exactly those operands in place of its own quantised values.  Then
      * the layer's output must agree to float accumulation level (bar 2e-3 on states of magnitude 3), so a wrong
        scale, layout, operand order or epilogue anywhere between two quantisers fails;
      * every device code must be a valid rounding of the value the oracle computed from the same upstream operands:
        equal to the oracle's own code or its neighbour on the e4m3 grid (saturation at 448 included: both follow the
        same rule; small elements of the attention output, whose bf16 softmax weights give it an absolute error of 2^-8
        of the row maximum, may be further off in steps, not in value), at most 15 % of them different (measured 8 % for the attention output, which passes through a bf16
        rounding on the device, a fraction of a per cent elsewhere), and without bias: the mean signed relative
        difference between the device's and the oracle's dequantised rows stays below 1 % (a 5 % error in the SwiGLU
        or norm arithmetic moves most elements to the neighbouring code in ONE direction and shifts that mean by 5 %).
    The wide shape (ffn_hidden 4096, heads x head_dim = 512) takes the decode-row kernels of full-size models: every
    projection as K-split row tiles, SwiGLU and the quantiser of the down projection's operand in the gate/up
    product's epilogue, the attention output quantised by the attention kernel; its states are larger, and the
    output bar scales with them."""
    from tests.helpers import oshape
    L, nl, d = shape.n_loops, shape.n_layers, shape.d_model
    weights = lively_weights(shape, 9, bf16=True, std=0.05)
    cfg = B.make_config(shape, dtype=B.PLT_BF16, w_dtype=B.PLT_MXFP4)
    model = B.Model(cfg, B.pack_weights(cfg, weights))
    Bn, n = 2, 9
    kv = B.KV(model, Bn, 20)
    prompts = synth.token_ids((Bn, n), shape.vocab, 10)
    nxt, _ = kv.prefill(torch.from_numpy(np.ascontiguousarray(prompts, np.int32)).cuda())
    nxt = nxt.cpu().numpy()
    pos = n
    carry = kv.get_carry()
    orcs = []
    for b in range(Bn):
        orc = O.PLTOracle(oshape(shape), weights, kv_bf16=True, w_mx=True)
        orc.kv = O.RingKV(orc._store, oshape(shape), pos + 1)
        for m in range(nl):
            e = kv.export(b, m, pos)
            orc.kv.ks[m, :pos] = e["k_share"].transpose(1, 0, 2); orc.kv.vs[m, :pos] = e["v_share"].transpose(1, 0, 2)
            for l in range(L - 1):
                orc.kv.kr[l, m] = e["k_ring"][l].transpose(1, 0, 2); orc.kv.vr[l, m] = e["v_ring"][l].transpose(1, 0, 2)
        orc.carry = carry[b].astype(np.float64).copy(); orc.pos = pos; orc.trace = []
        orc.layer_trace = []
        orc.clp_decode_step(int(nxt[b]))                      # free run: the layer inputs to teacher-force with
        orc.x_in = {(l, m): a for (l, m, p, a, _) in orc.layer_trace}
        orcs.append(orc)

    def dequant(codes, scales, K):
        blk = np.arange(K // 32)
        sidx = (blk >> 4) * 16 + (blk & 3) * 4 + ((blk >> 2) & 3)                  # plt_mx_act_scale_index
        ex = scales[:, sidx].astype(np.int64) - 127                                # [rows, K/32]
        return synth.e4m3_from_bits(codes).astype(np.float64) * np.repeat(np.ldexp(1.0, ex), 32, axis=1), ex

    worst_out, worst_bias, n_elem, n_diff, top_out = 0.0, 0.0, 0, 0, 0.0
    for m in range(nl):
        kv.set_position(pos)
        xin = np.zeros((Bn, L, d), np.float32)
        for b in range(Bn):
            for l in range(1, L + 1):
                xin[b, l - 1] = orcs[b].x_in[(l, m)]
        out = kv.debug_layer(m, xin)
        stages = []
        for st in range(4):
            codes, scales = kv.debug_act_codes(st)
            stages.append(dequant(codes, scales, codes.shape[1]))
        for b in range(Bn):
            orc = orcs[b]
            orc.act_override = {(l, m, st): stages[st][0][b * L + l - 1] for l in range(1, L + 1) for st in range(4)}
            orc.act_trace = []
            for l in range(1, L + 1):
                ref = orc.f(xin[b, l - 1].astype(np.float64), pos, l, orc.kv, layers=[m])
                worst_out = max(worst_out, float(np.max(np.abs(out[b, l - 1] - ref))))
                top_out = max(top_out, float(np.max(np.abs(ref))))
            for (l, mm, st, t) in orc.act_trace:
                dev, ex = stages[st][0][b * L + l - 1], stages[st][1][b * L + l - 1]
                q_own, e_own = O.mx_quantize(t, "e4m3")
                own = O.mx_dequantize(q_own, e_own)
                same_scale = np.repeat(e_own == ex, 32)
                # one grid step at the element's magnitude (2^-3 of its binade; 2^-9 of the block scale for subnormals)
                mag = np.maximum(np.abs(own), np.abs(dev)) / np.repeat(np.ldexp(1.0, e_own), 32)
                step = np.ldexp(1.0, np.maximum(np.floor(np.log2(np.maximum(mag, 2.0 ** -20))), -6).astype(np.int64) - 3) * np.repeat(np.ldexp(1.0, e_own), 32)
                # the attention output reaches its quantiser through bf16 softmax weights and a bf16 store: an ABSOLUTE
                # error of 2^-8 of the row's largest entry, which moves small elements by more than one of their steps
                slack = (2.0 ** -8 if st == 1 else 2.0 ** -12) * float(np.max(np.abs(t)))
                ok = np.where(same_scale, np.abs(dev - own) <= step * (1 + 1e-9) + slack, np.abs(dev - t) <= 2.0 ** -3 * np.abs(t) + step + slack)
                assert np.all(ok), (m, b, l, st, np.where(~ok)[0][:8], dev[~ok][:8], own[~ok][:8], t[~ok][:8])
                n_elem += dev.size; n_diff += int(np.sum(dev != own))
                big = np.abs(own) > 0.05 * np.max(np.abs(own))
                worst_bias = max(worst_bias, abs(float(np.mean((dev[big] - own[big]) / own[big]))))
            orc.act_override = None
    print(f"layer outputs from the device's own codes: max-abs {worst_out:.2e} (largest |output| {top_out:.2f}); codes that are the oracle's neighbour: {n_diff} of {n_elem}; "
          f"largest mean signed deviation of a quantised row {worst_bias:.2e}")
    assert worst_out <= 2e-3 * max(1.0, top_out / 3.0) and worst_bias <= 1e-2 and n_diff <= 0.15 * n_elem, (worst_out, top_out, worst_bias, n_diff, n_elem)
    kv.close(); model.close()
