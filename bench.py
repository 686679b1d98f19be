#!/usr/bin/env python3
"""Benchmark of the PLT cross-loop-parallel decode step on one MI355X.

Headline workload ("c3"): one full CLP decode step of the ~1.3B dense PLT in bf16 -- 24 layers,
d_model 2048, 16 heads of 128, SwiGLU 5632, vocab 32000, L = 2, window 64, batch 64, 2048-token
shared KV context -- all inputs synthetic and seeded, resident in HBM before the timed region.
A "step" is one plt_decode_step over the whole batch (every stage of the hot path, one new
token per sequence).  Prints ONE JSON line (see the keys below); extra keys carry the
non-looped / vanilla-loop / L-sweep latencies, the kernel-only attention configuration and the
CPU oracle timed on the host cores.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--only-main] [--no-cpu-baseline]

Single-section runs for profiling (each prints its own JSON line): --attn-kernel-only, --prefill-only, --prefill-moe-only,
--copy-reference; --kv-fp8 runs the main workload with e4m3 K/V caches (a labelled variant, not the
headline).
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
SEED = 2510


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def fill_weights_on_device(B, cfg, seed):
    """N(0, 0.02) weights drawn on the device straight into the library's blob layout
    (norm gains 1, gate bias 0); returns the uint8 blob tensor."""
    import torch
    nbytes = B.lib().plt_weights_bytes(C.byref(cfg))
    blob = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    g = torch.Generator(device="cuda"); g.manual_seed(seed)

    def view(layer, which, dtype):
        off, n = B.weights_offset(cfg, layer, which)
        es = 2 if dtype == torch.bfloat16 else 4
        return blob[off:off + es * n].view(dtype), n

    def normal(layer, which, dtype):
        v, n = view(layer, which, dtype)
        step = 1 << 26
        for i in range(0, n, step):
            m = min(step, n - i)
            v[i:i + m].copy_((torch.randn(m, generator=g, device="cuda") * 0.02).to(dtype))

    wd = torch.bfloat16 if cfg.dtype == B.PLT_BF16 else torch.float32
    Hq, Hkv, D, d, F = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_model, cfg.ffn_hidden

    def matrix(layer, which, which_sc, N, K, count=1):
        if cfg.w_dtype == B.PLT_MXFP4:      # low-bit projections: a bf16 draw quantised on the device into the blob
            for index in range(count):
                w = (torch.randn(N, K, generator=g, device="cuda") * 0.02).to(torch.bfloat16)
                B.quantize_into_blob(cfg, blob, layer, which, which_sc, w, index)
        else:
            normal(layer, which, wd)

    normal(0, B.PLT_W_EMB, wd)
    for m in range(cfg.n_layers):
        view(m, B.PLT_W_NORM1, torch.float32)[0].fill_(1.0)
        matrix(m, B.PLT_W_WQKV, B.PLT_W_WQKV_SC, (Hq + 2 * Hkv) * D, d)
        normal(m, B.PLT_W_GATE_W, torch.float32)
        matrix(m, B.PLT_W_WO, B.PLT_W_WO_SC, d, Hq * D)
        view(m, B.PLT_W_NORM2, torch.float32)[0].fill_(1.0)
        if cfg.n_experts > 0:
            normal(m, B.PLT_W_ROUTER, wd)
            matrix(m, B.PLT_W_WGU, B.PLT_W_WGU_SC, 2 * F, d, cfg.n_experts)
            matrix(m, B.PLT_W_WDOWN, B.PLT_W_WDOWN_SC, d, F, cfg.n_experts)
        else:
            matrix(m, B.PLT_W_WGU, B.PLT_W_WGU_SC, 2 * F, d)
            matrix(m, B.PLT_W_WDOWN, B.PLT_W_WDOWN_SC, d, F)
    view(0, B.PLT_W_NORM_F, torch.float32)[0].fill_(1.0)
    if not cfg.tie_embeddings:
        normal(0, B.PLT_W_HEAD, wd)
    return blob


def with_layers(shape, n_layers):
    """The same per-layer shape at another depth."""
    import dataclasses
    return dataclasses.replace(shape, n_layers=n_layers)


def moe_untile(t):
    """Inverse of the blob's strip order of bf16 expert matrices (binding.moe_tile_weights): [..., N, K] row-major."""
    *lead, N, K = t.shape
    nl = len(lead)
    x = t.reshape(*lead, N // 16, K // 32, 4, 16, 8)
    x = np.transpose(x, tuple(range(nl)) + (nl, nl + 3, nl + 1, nl + 2, nl + 4))
    return np.ascontiguousarray(x).reshape(*lead, N, K)


def weights_to_host(B, cfg, blob):
    """The device blob as the float32 weight dict the oracle takes (same values)."""
    import torch
    wd = torch.bfloat16 if cfg.dtype == B.PLT_BF16 else torch.float32
    Hq, Hkv, D, d, F = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_model, cfg.ffn_hidden

    def get(layer, which, dtype, shape):
        off, n = B.weights_offset(cfg, layer, which)
        es = 2 if dtype == torch.bfloat16 else 4
        return blob[off:off + es * n].view(dtype).float().cpu().numpy().reshape(shape)

    w = {"emb": get(0, B.PLT_W_EMB, wd, (cfg.vocab, d)), "norm_f": get(0, B.PLT_W_NORM_F, torch.float32, (d,)), "layers": []}
    if not cfg.tie_embeddings:
        w["head"] = get(0, B.PLT_W_HEAD, wd, (cfg.vocab, d))
    E = cfg.n_experts
    for m in range(cfg.n_layers):
        qkv = get(m, B.PLT_W_WQKV, wd, ((Hq + 2 * Hkv) * D, d))
        if E > 0:
            untile = moe_untile if cfg.dtype == B.PLT_BF16 else (lambda x: x)
            gu = untile(get(m, B.PLT_W_WGU, wd, (E, 2 * F, d)))
            w["layers"].append({
                "norm1": get(m, B.PLT_W_NORM1, torch.float32, (d,)), "wq": qkv[:Hq * D], "wk": qkv[Hq * D:(Hq + Hkv) * D],
                "wv": qkv[(Hq + Hkv) * D:], "gate_w": get(m, B.PLT_W_GATE_W, torch.float32, (Hq, D)),
                "gate_b": get(m, B.PLT_W_GATE_B, torch.float32, (Hq,)), "wo": get(m, B.PLT_W_WO, wd, (d, Hq * D)),
                "norm2": get(m, B.PLT_W_NORM2, torch.float32, (d,)), "router": get(m, B.PLT_W_ROUTER, wd, (E, d)),
                "w_gate": gu[:, :F], "w_up": gu[:, F:], "w_down": untile(get(m, B.PLT_W_WDOWN, wd, (E, d, F)))})
            continue
        gu = get(m, B.PLT_W_WGU, wd, (2 * F, d))
        w["layers"].append({
            "norm1": get(m, B.PLT_W_NORM1, torch.float32, (d,)), "wq": qkv[:Hq * D], "wk": qkv[Hq * D:(Hq + Hkv) * D],
            "wv": qkv[(Hq + Hkv) * D:], "gate_w": get(m, B.PLT_W_GATE_W, torch.float32, (Hq, D)),
            "gate_b": get(m, B.PLT_W_GATE_B, torch.float32, (Hq,)), "wo": get(m, B.PLT_W_WO, wd, (d, Hq * D)),
            "norm2": get(m, B.PLT_W_NORM2, torch.float32, (d,)), "w_gate": gu[:F], "w_up": gu[F:],
            "w_down": get(m, B.PLT_W_WDOWN, wd, (d, F))})
    return w


def attn_alg_bytes(Bn, L, Hq, Hkv, D, N, w, es=2, kes=None):
    """Algorithmic HBM bytes of one fused decode-attention launch: shared K and V once, the
    rings once, Q in, Y out (es: bytes per q / y element, kes: per cache element)."""
    kes = es if kes is None else kes
    share = 2 * Bn * Hkv * N * D * kes
    ring = 2 * Bn * (L - 1) * Hkv * min(w, N) * D * kes
    qy = 2 * Bn * L * Hq * D * es
    return share + ring + qy


def fill_kv_random(B, kv, g, std=0.5):
    """Timing-only cache contents drawn on the device: N(0, std) in the cache's element type."""
    import torch
    if kv.model.cfg.kv_dtype == B.PLT_FP8_E4M3:
        step = 1 << 28
        for i in range(0, kv.buf.numel(), step):
            m = min(step, kv.buf.numel() - i)
            kv.buf[i:i + m].copy_((torch.randn(m, generator=g, device="cuda", dtype=torch.bfloat16) * std)
                                  .to(torch.float8_e4m3fn).view(torch.uint8))
    else:
        kv.buf.view(torch.bfloat16).normal_(0.0, std, generator=g)


def time_steps(kv, pos, tok, warmup, steps):
    import torch
    for _ in range(warmup):
        kv.set_position(pos)
        kv.decode_step(tok, want_logits=False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        kv.set_position(pos)
        kv.decode_step(tok, want_logits=False)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def copy_reference(B):
    """Four launches of the library's plain copy kernel, 1 GiB read + 1 GiB written each: the known-size
    reference that scales rocprofv3's FETCH_SIZE / WRITE_SIZE readings."""
    import torch
    n = 1 << 30
    a = torch.zeros(n, dtype=torch.uint8, device="cuda"); b = torch.zeros(n, dtype=torch.uint8, device="cuda")
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    assert B.lib().plt_stream_copy(C.c_void_p(b.data_ptr()), C.c_void_p(a.data_ptr()), n, stream) == 0
    e0.record()
    for _ in range(3):
        assert B.lib().plt_stream_copy(C.c_void_p(b.data_ptr()), C.c_void_p(a.data_ptr()), n, stream) == 0
    e1.record(); torch.cuda.synchronize()
    return {"workload": "k_stream_copy, 4 launches, 1 GiB read + 1 GiB written each", "bytes_read_per_launch": n,
            "bytes_written_per_launch": n, "GBps_read_plus_write": 2 * n / (e0.elapsed_time(e1) * 1e-3 / 3) / 1e9}


def oracle_sample(B, shape, cfg, blob, state, pos, gpu_logits, gpu_hidden, gpu_next, kv=None):
    """One decode step of each sampled sequence through the CPU oracle, from the exported device
    state.  state: {seq: (exports per layer, carry, token)}; gpu_*: {seq: array}.  With kv (the device object,
    still alive): additionally every layer of the device is fed the oracle's input of that layer for the sampled
    sequences (plt_debug_layer) and the largest |device - oracle| of any layer's output rows is reported: the
    per-layer, teacher-forced parity, free of the accumulation of bf16 roundings over depth."""
    from oracle import plt_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = 1
    w = weights_to_host(B, cfg, blob)
    osh = O.OracleShape(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim,
                        shape.ffn_hidden, shape.vocab, cfg.n_loops, cfg.window, shape.rope_theta, shape.norm_eps,
                        shape.tie_embeddings)
    total, err_l, err_h, rel_h, same = 0.0, 0.0, 0.0, 0.0, True
    layer_io = {}
    for seq, (exports, carry0, token0) in state.items():
        fp8 = cfg.kv_dtype == B.PLT_FP8_E4M3
        orc = O.PLTOracle(osh, w, kv_bf16=not fp8, kv_fp8=fp8)
        orc.kv = O.RingKV(orc._store, osh, pos + 1)
        for m, e in enumerate(exports):
            orc.kv.ks[m, :pos] = e["k_share"].transpose(1, 0, 2); orc.kv.vs[m, :pos] = e["v_share"].transpose(1, 0, 2)
            for l in range(cfg.n_loops - 1):
                orc.kv.kr[l, m] = e["k_ring"][l].transpose(1, 0, 2); orc.kv.vr[l, m] = e["v_ring"][l].transpose(1, 0, 2)
        orc.carry = carry0.astype(np.float64).copy(); orc.pos = pos; orc.trace = []; orc.layer_trace = []
        t0 = time.perf_counter()
        nxt, lg = orc.clp_decode_step(int(token0))
        total += time.perf_counter() - t0
        x_in = np.zeros((cfg.n_loops, shape.n_layers, shape.d_model)); x_out = np.zeros_like(x_in)
        for (l, m, p, a, b) in orc.layer_trace:
            x_in[l - 1, m] = a; x_out[l - 1, m] = b
        layer_io[seq] = (x_in, x_out)
        err_l = max(err_l, float(np.max(np.abs(lg - gpu_logits[seq]))))
        err_h = max(err_h, float(np.max(np.abs(orc.trace[-1] - gpu_hidden[seq]))))
        rel_h = max(rel_h, float(np.max(np.abs(orc.trace[-1] - gpu_hidden[seq])) / np.max(np.abs(orc.trace[-1]))))
        top2 = np.sort(lg)[-2:]
        if top2[1] - top2[0] > 2 * 2e-2:          # away from a near-tie the greedy id must agree
            same = same and (nxt == gpu_next[seq])
    n = len(state)
    out = {"value": n / total, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
           "sample": f"{n} of the batch's {cfg_batch_note(state)} sequences, one decode step each (all {cfg.n_loops} loop rows, "
                     f"{shape.n_layers} layers, context {pos + 1}) from the device's exported KV state; {total:.1f} s of CPU work",
           "seconds": total, "parity_max_abs_logits": err_l,
           "accumulated_hidden_drift_max_abs": err_h, "accumulated_hidden_drift_max_rel": rel_h,
           "accumulated_hidden_drift_note": f"free-running residual stream after all {shape.n_layers} layers (bf16 roundings add up over depth); "
                                            "the parity bar is held per layer, see parity_per_layer_teacher_forced_max_abs",
           "greedy_ids_equal_where_margin_gt_0.04": bool(same)}
    if kv is not None:
        worst = 0.0
        for m in range(shape.n_layers):
            kv.set_position(pos)
            xin = np.zeros((kv.batch, cfg.n_loops, shape.d_model), np.float32)
            for seq, (x_in, _) in layer_io.items():
                xin[seq] = x_in[:, m]
            got = kv.debug_layer(m, xin)
            for seq, (x_in, x_out) in layer_io.items():
                ref = x_out[:, m] - x_in[:, m] + xin[seq].astype(np.float64)
                worst = max(worst, float(np.max(np.abs(got[seq] - ref))))
        out["parity_per_layer_teacher_forced_max_abs"] = worst
    return out


def cfg_batch_note(state):
    return "sampled (" + ",".join(str(k) for k in state) + ")"


def bench_attn_kernel(B, steps, warmup, fp8=False):
    """Kernel-only fused decode attention: batch 32, L=3, 16 q / 4 kv heads, D=128, 4096 keys, w=64.
    Four disjoint input sets are rotated so that a launch never finds its KV in the 256 MB last-level cache.
    fp8: the four cache arrays hold e4m3 bytes (q, y stay bf16); eight sets are rotated then."""
    import torch
    Bn, L, Hq, Hkv, D, N, w = 32, 3, 16, 4, 128, 4096, 64
    g = torch.Generator(device="cuda"); g.manual_seed(SEED + 2)
    rn = lambda *s: torch.randn(*s, generator=g, device="cuda").to(torch.bfloat16)
    rc = (lambda *s: rn(*s).to(torch.float8_e4m3fn).view(torch.uint8)) if fp8 else rn
    dt = B.PLT_FP8_E4M3 if fp8 else B.PLT_BF16
    n_sets = 8 if fp8 else 4
    sets = []
    for _ in range(n_sets):
        sets.append(dict(q=rn(Bn, L, Hq, D), ks=rc(Bn, Hkv, N, D), vs=rc(Bn, Hkv, N // 32, D, 32),
                         kr=rc(Bn, L - 1, Hkv, w, D), vr=rc(Bn, L - 1, Hkv, w // 32, D, 32),
                         z=torch.randn(Bn, L - 1, Hq, generator=g, device="cuda"), y=torch.empty(Bn, L, Hq, D, dtype=torch.bfloat16, device="cuda")))
    nb = B.lib().plt_attn_scratch_bytes(Bn, L, Hq, Hkv, D)
    scratch = torch.zeros(nb, dtype=torch.uint8, device="cuda")
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda t: C.c_void_p(t.data_ptr())

    def launch(s):
        st = B.lib().plt_attn_decode(dt, Bn, L, Hq, Hkv, D, N, N, w, w, p(s["q"]), p(s["ks"]), p(s["vs"]), p(s["kr"]),
                                     p(s["vr"]), p(s["z"]), p(s["y"]), p(scratch), nb, 0, stream)
        if st:
            raise RuntimeError(B.lib().plt_last_error().decode())

    for i in range(warmup):
        launch(sets[i % n_sets])
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n = max(steps, 8) * 4
    e0.record()
    for i in range(n):
        launch(sets[i % n_sets])
    e1.record(); torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / n
    nbytes = attn_alg_bytes(Bn, L, Hq, Hkv, D, N, w, 2, 1 if fp8 else 2)
    gbs = nbytes / (us * 1e-6) / 1e9
    return {"workload": f"fused decode attention, {'bf16 q/y + e4m3 caches' if fp8 else 'bf16'}, B=32, L=3, 16q/4kv heads, D=128, N=4096, w=64",
            "us_per_launch": us, "algorithmic_bytes": nbytes, "achieved_GBps": gbs, "frac_of_8TBps": gbs / HBM_PEAK_GBS,
            "launches_timed": n}


def bench_long_context(B, shape, blob, g, steps, parity=True):
    """L = 4, window 128, 8192-token shared KV (the KV-bandwidth-bound configuration, configs[3]).  Batch 256 needs
    412 GB of shared KV in bf16 and does not fit one GPU.  What one GPU shows:
      * batch 128 (206 GB + 9.7 GB of windows), resident, PLT L = 4 against the non-looped model; the PLT state is built
        by plt_prefill of 128 x 8191 tokens and one sampled sequence's step is checked against the oracle (logits end
        to end, every layer teacher-forced);
      * batch 256 at the real per-layer shape with the shared caches of 12 layers in memory, aliased to the 24 layers
        (timing only: each layer still streams its full 17 GB, so the bytes moved are the real ones);
      * the vanilla sequential loop keeps 4 full caches, so it is timed at batch 32 (the same 206 GB) per sequence;
      * with e4m3 caches the whole batch-256 configuration is resident (206 GB + 4.8 GB of windows).
    Caches of the timing-only rows hold N(0, 0.5) values drawn on the device."""
    import torch
    N, w = 8192, 128
    pos = N - 1
    res = {"context": N, "window": w, "workload": "~1.3B PLT, bf16, L=4, window 128, 8192-token shared KV (configs[3]); batch 256 = 412 GB of KV "
                                                   "exceeds 288 GB: batch 128 resident (parity-checked), batch 256 with 12 of 24 layers of shared cache in "
                                                   "memory (aliased, timing only), batch 256 resident with e4m3 caches"}
    rows = [("plt_L4_b128", B.PLT_MODE_CLP, 4, 128, 0, 0), ("nonlooped_L1_b128", B.PLT_MODE_CLP, 1, 128, 0, 0),
            ("plt_L4_b32", B.PLT_MODE_CLP, 4, 32, 0, 0), ("vanilla_loop_L4_b32", B.PLT_MODE_VANILLA_LOOP, 4, 32, 0, 0),
            ("plt_L4_b256_aliased", B.PLT_MODE_CLP, 4, 256, 0, 12), ("nonlooped_L1_b256_aliased", B.PLT_MODE_CLP, 1, 256, 0, 12),
            ("plt_L4_b256_fp8kv", B.PLT_MODE_CLP, 4, 256, B.PLT_FP8_E4M3, 0),
            ("nonlooped_L1_b256_fp8kv", B.PLT_MODE_CLP, 1, 256, B.PLT_FP8_E4M3, 0)]
    for name, mode, Lx, Bn, kvd, alias in rows:
        cfg = B.make_config(shape, dtype=B.PLT_BF16, mode=mode, n_loops=Lx, window=w, kv_dtype=kvd)
        m = B.Model(cfg, blob)
        m.kv_alias_layers(alias)
        kv = B.KV(m, Bn, N)
        tok = torch.randint(0, shape.vocab, (Bn,), generator=g, device="cuda", dtype=torch.int32)
        row = {}
        if name == "plt_L4_b128" and parity:
            # real state + the parity leg of this configuration
            t0 = time.perf_counter()
            prompt = torch.randint(0, shape.vocab, (Bn, pos), generator=g, device="cuda", dtype=torch.int32)
            nxt, _ = kv.prefill(prompt, want_logits=False)
            torch.cuda.synchronize()
            row["kv_fill"] = f"plt_prefill of {Bn} x {pos} uniform token ids ({time.perf_counter() - t0:.1f} s)"
            kv.drop_workspace(); del prompt
            b = 77
            carry_all = kv.get_carry()
            state = {b: ([kv.export(b, l, pos) for l in range(shape.n_layers)], carry_all[b], int(nxt[b].item()))}
            tok = nxt.clone()
            n1, lg1 = kv.decode_step(tok)
            hid1 = kv.get_hidden()
            row["parity"] = oracle_sample(B, shape, cfg, blob, state, pos, {b: lg1[b].float().cpu().numpy().astype(np.float64)},
                                          {b: hid1[b].astype(np.float64)}, {b: int(n1[b].item())}, kv=kv)
            log(f"[bench] long context parity (batch 128, sequence {b}): logits {row['parity']['parity_max_abs_logits']:.2e}, "
                f"per layer {row['parity']['parity_per_layer_teacher_forced_max_abs']:.2e}")
        else:
            fill_kv_random(B, kv, g)
            row["kv_fill"] = "N(0, 0.5) drawn on the device (timing only)" + (f"; shared caches of {alias} layers aliased to {shape.n_layers}" if alias else "")
        m.profile_enable(1 << B.PLT_PROF_ATTN)
        ms = time_steps(kv, pos, tok, 1, steps)
        attn_ms, attn_n = m.profile_read(B.PLT_PROF_ATTN, reset=True)
        ab = attn_alg_bytes(Bn, Lx if mode == B.PLT_MODE_CLP else 1, shape.n_heads, shape.n_kv_heads, shape.head_dim, N, w,
                            2, 1 if kvd else 2)
        us = attn_ms * 1e3 / max(attn_n, 1)
        row.update({"ms_per_step": ms, "tokens_per_s": Bn / (ms * 1e-3), "attn_us_per_launch": us,
                    "attn_GBps": ab / (us * 1e-6) / 1e9, "attn_frac_of_8TBps": ab / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                    "kv_bytes": m.kv_logical_bytes(Bn, N)})
        res[name] = row
        log(f"[bench] long context {name}: {ms:.2f} ms/step, attention {us:.0f} us/launch = {ab / (us * 1e-6) / 1e12:.2f} TB/s")
        kv.close(); m.close(); del kv
        torch.cuda.empty_cache()
    res["latency_plt_L4_vs_nonlooped_b128"] = res["plt_L4_b128"]["ms_per_step"] / res["nonlooped_L1_b128"]["ms_per_step"]
    res["latency_vanilla_L4_vs_plt_L4_b32"] = res["vanilla_loop_L4_b32"]["ms_per_step"] / res["plt_L4_b32"]["ms_per_step"]
    res["latency_plt_L4_vs_nonlooped_b256_aliased"] = (res["plt_L4_b256_aliased"]["ms_per_step"]
                                                       / res["nonlooped_L1_b256_aliased"]["ms_per_step"])
    res["latency_plt_L4_vs_nonlooped_b256_fp8kv"] = (res["plt_L4_b256_fp8kv"]["ms_per_step"]
                                                      / res["nonlooped_L1_b256_fp8kv"]["ms_per_step"])
    return res


def bench_prefill(B, shape, blob, g, Bn=4, n=8192, L=3, w=64, reps=2):
    """CLP prefill / forward (Alg. 2) of Bn prompts of n uniform token ids at L loops: all loops with the
    cross-loop shift in one call.  MFMA-bound (projections + causal attention); flops counted as
    2 * params * tokens * L for the projections plus 4 * D * (n^2/2 + (L-1)/L * n * w) per head and loop
    for the attention.  Returns time, tokens/s and the matrix-core roofline fraction."""
    import torch
    cfg = B.make_config(shape, dtype=B.PLT_BF16, n_loops=L, window=w)
    m = B.Model(cfg, blob)
    kv = B.KV(m, Bn, n + 1)
    prompt = torch.randint(0, shape.vocab, (Bn, n), generator=g, device="cuda", dtype=torch.int32)
    kv.prefill(prompt, want_logits=False); torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        kv.prefill(prompt, want_logits=False)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    # feed-forward weights a row multiplies: the dense SwiGLU, or (mixture of experts) the router and top_k experts
    ffn = 3 * shape.ffn_hidden * shape.d_model
    if shape.n_experts:
        ffn = shape.top_k * ffn + shape.n_experts * shape.d_model
    params = shape.n_layers * ((shape.n_heads + 2 * shape.n_kv_heads) * shape.head_dim * shape.d_model
                               + shape.d_model * shape.n_heads * shape.head_dim + ffn)
    fl_gemm = 2.0 * params * Bn * n * L + 2.0 * shape.vocab * shape.d_model * Bn
    fl_attn = 4.0 * shape.head_dim * shape.n_heads * Bn * shape.n_layers * (L * n * n / 2 + (L - 1) * n * min(w, n))
    kv.close(); m.close(); del kv
    torch.cuda.empty_cache()
    tf = (fl_gemm + fl_attn) / dt / 1e12
    what = (f"{shape.top_k}-of-{shape.n_experts} mixture-of-experts shape" if shape.n_experts else "~1.3B PLT")
    return {"workload": f"CLP prefill, {what}, bf16, L={L}, window {w}, batch {Bn}, {n}-token prompts" + ("" if shape.n_experts else " (configs[4])"),
            "ms": dt * 1e3, "tokens_per_s": Bn * n / dt, "flops_projections": fl_gemm, "flops_attention": fl_attn,
            "roofline": {"bound": "mfma", "achieved": tf, "peak": 2500.0, "unit": "TFLOP/s", "frac": tf / 2500.0, "traffic": None}}


def bench_sweep(B, shape, blob, g, n_new=256, runs=5, contexts=(1024, 2048, 5000), batches=(1, 4, 16, 64, 256), graph=True):
    """The paper's serving recipe on synthetic inputs: prefill context {1024, 2048, 5000}, batch 1..256,
    n_new consecutive greedy decode steps (the context grows), mean per-token latency over `runs` runs,
    for the non-looped model, PLT-2 and the vanilla sequential loop-2 in the same library.  Caches are
    filled with N(0, 0.5) values on the device (timing only)."""
    import torch
    free_bytes = torch.cuda.mem_get_info()[0]
    table = []
    torch.cuda.synchronize()
    side = torch.cuda.Stream()          # stream capture needs a stream of its own; default priority
    with torch.cuda.stream(side):
        _sweep_rows(B, shape, blob, g, n_new, runs, contexts, batches, graph, free_bytes, table)
    torch.cuda.synchronize()
    return {"decoded_tokens": n_new, "runs": runs, "unit": "ms per token", "step_replayed_as_hip_graph": bool(graph), "rows": table}


def _sweep_rows(B, shape, blob, g, n_new, runs, contexts, batches, graph, free_bytes, table):
    import torch
    for ctx in contexts:
        for bs in batches:
            row = {"context": ctx, "batch": bs}
            for name, mode, Lx in [("nonlooped", B.PLT_MODE_CLP, 1), ("plt2", B.PLT_MODE_CLP, 2), ("vanilla_loop2", B.PLT_MODE_VANILLA_LOOP, 2)]:
                cfg = B.make_config(shape, dtype=B.PLT_BF16, mode=mode, n_loops=Lx, window=64)
                m = B.Model(cfg, blob)
                m.use_graph(graph)
                need = m.kv_bytes(bs, ctx + n_new)
                if need > free_bytes - (8 << 30):
                    row[name] = None
                    m.close()
                    continue
                kv = B.KV(m, bs, ctx + n_new)
                kv.buf.view(torch.bfloat16).normal_(0.0, 0.5, generator=g)
                tok = torch.randint(0, shape.vocab, (bs,), generator=g, device="cuda", dtype=torch.int32)
                ms = []
                for r in range(runs + 1):
                    kv.set_position(ctx)
                    nxt = tok
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    for _ in range(n_new):
                        nxt, _ = kv.decode_step(nxt, want_logits=False)
                    torch.cuda.synchronize()
                    if r > 0:                       # run 0 warms up
                        ms.append((time.perf_counter() - t0) * 1e3 / n_new)
                row[name] = sum(ms) / len(ms)
                kv.close(); m.close(); del kv
                torch.cuda.empty_cache()
            if row["nonlooped"]:
                row["plt2_vs_nonlooped"] = row["plt2"] / row["nonlooped"] if row["plt2"] else None
                row["vanilla_loop2_vs_nonlooped"] = row["vanilla_loop2"] / row["nonlooped"] if row["vanilla_loop2"] else None
            log(f"[bench] sweep {row}")
            table.append(row)


def bench_sweep_moe(B, g, n_new=256, runs=5, ctx=5000):
    """The protocol of the paper's mixture-of-experts latency table on synthetic inputs: prefill context 5000,
    batch 4..64, 256 consecutive greedy decode steps, mean per-token latency over 5 runs, with the serving
    formats (here: e4m3 caches, MXFP4 projections and experts) -- on the open-source 8-of-64 recipe's shape, for
    the non-looped model, PLT-2, PLT-3 and the vanilla sequential loop-2.  Caches hold N(0, 0.5) values."""
    import torch
    from paper_2510_24824_amd import synth
    shape = synth.PLT_MOE_1B7B
    blob = fill_weights_on_device(B, B.make_config(shape, dtype=B.PLT_BF16, w_dtype=B.PLT_MXFP4), SEED + 7)
    table = []
    for bs in (4, 8, 16, 32, 64):
        row = {"context": ctx, "batch": bs}
        for name, mode, Lx in [("nonlooped", B.PLT_MODE_CLP, 1), ("plt2", B.PLT_MODE_CLP, 2), ("plt3", B.PLT_MODE_CLP, 3),
                               ("vanilla_loop2", B.PLT_MODE_VANILLA_LOOP, 2)]:
            cfg = B.make_config(shape, dtype=B.PLT_BF16, mode=mode, n_loops=Lx, window=64, kv_dtype=B.PLT_FP8_E4M3, w_dtype=B.PLT_MXFP4)
            m = B.Model(cfg, blob)
            kv = B.KV(m, bs, ctx + n_new)
            fill_kv_random(B, kv, g)
            tok = torch.randint(0, shape.vocab, (bs,), generator=g, device="cuda", dtype=torch.int32)
            ms = []
            for r in range(runs + 1):
                kv.set_position(ctx)
                nxt = tok
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(n_new):
                    nxt, _ = kv.decode_step(nxt, want_logits=False)
                torch.cuda.synchronize()
                if r > 0:                       # run 0 warms up
                    ms.append((time.perf_counter() - t0) * 1e3 / n_new)
            row[name] = sum(ms) / len(ms)
            kv.close(); m.close(); del kv
            torch.cuda.empty_cache()
        for k in ("plt2", "plt3", "vanilla_loop2"):
            row[k + "_vs_nonlooped"] = row[k] / row["nonlooped"]
        log(f"[bench] MoE sweep {row}")
        table.append(row)
    return {"decoded_tokens": n_new, "runs": runs, "unit": "ms per token", "rows": table,
            "workload": "8-of-64 MoE shape, e4m3 caches + MXFP4 projections and experts"}


def bench_lowbit_gemm(B, Mrows=128, reps=30):
    """Kernel-only: the four per-layer projections of the 1.3B model as block-scaled low-bit GEMMs (MXFP4
    weights x MXFP8 activations) next to the bf16 decode GEMM, each timed over back-to-back calls that
    rotate through 8 weight copies (so that no call finds its weights in a cache), slab-sum kernel included."""
    import torch
    g = torch.Generator(device="cuda"); g.manual_seed(SEED + 9)
    l = B.lib()
    st = B._stream()

    def timed(fn):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record(); torch.cuda.synchronize()
        return a.elapsed_time(b) / reps * 1e3

    out = {"rows": Mrows, "projections": {}}
    for name, N, K in (("qkv", 6144, 2048), ("out", 2048, 2048), ("gate_up", 11264, 2048), ("down", 2048, 5632)):
        ws = [(torch.randn(N, K, generator=g, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(8)]
        x = torch.randn(Mrows, K, generator=g, device="cuda")
        xb = x.to(torch.bfloat16)
        q = [B.mx_quantize_weights(w) for w in ws]
        ac, asc = B.mx_quantize_act(x)
        c = torch.empty(Mrows, N, device="cuda")
        nb1 = l.plt_gemm_mx_scratch_bytes(Mrows, N, K); s1 = torch.empty(nb1, dtype=torch.uint8, device="cuda")
        nb2 = l.plt_gemm_scratch_bytes(Mrows, N, K); s2 = torch.empty(nb2, dtype=torch.uint8, device="cuda")
        i = [0]

        def run_mx():
            wc, wsc = q[i[0] % 8]; i[0] += 1
            B._check(l.plt_gemm_mx(Mrows, N, K, B._ptr(ac), B._ptr(asc), B._ptr(wc), B._ptr(wsc), B._ptr(c), B._ptr(s1), nb1, st))

        def run_bf():
            w = ws[i[0] % 8]; i[0] += 1
            B._check(l.plt_gemm(B.PLT_BF16, Mrows, N, K, B._ptr(xb), B._ptr(w), B._ptr(c), B._ptr(s2), nb2, st))

        def run_q():
            B._check(l.plt_mx_quantize_act(B.PLT_F32, Mrows, K, B._ptr(x), B._ptr(ac), B._ptr(asc), st))

        t_mx, t_bf, t_q = timed(run_mx), timed(run_bf), timed(run_q)
        out["projections"][name] = {"N": N, "K": K, "mxfp4_us": t_mx, "bf16_us": t_bf, "act_quant_us": t_q,
                                    "mx_weight_bytes": N * K // 2 + N * K // 32, "bf16_weight_bytes": N * K * 2}
        log(f"[bench] low-bit GEMM {name} {Mrows}x{N}x{K}: MXFP4 {t_mx:.1f} us, bf16 {t_bf:.1f} us, activation quantiser {t_q:.1f} us")
        if name == "gate_up":
            # as the model runs it: SwiGLU and the quantiser of the down projection's operand in the product's epilogue
            F = N // 2
            hc = torch.empty(Mrows, F, dtype=torch.uint8, device="cuda")
            hs = torch.empty(l.plt_mx_act_scale_bytes(Mrows, F), dtype=torch.uint8, device="cuda")
            nb3 = l.plt_gemm_mx_swiglu_scratch_bytes(Mrows, F, K); s3 = torch.empty(nb3, dtype=torch.uint8, device="cuda")

            def run_fused():
                wc, wsc = q[i[0] % 8]; i[0] += 1
                B._check(l.plt_gemm_mx_swiglu(Mrows, F, K, B._ptr(ac), B._ptr(asc), B._ptr(wc), B._ptr(wsc), B._ptr(hc), B._ptr(hs),
                                              B._ptr(s3), nb3, st))

            t_f = timed(run_fused)
            out["projections"][name]["mxfp4_swiglu_quantiser_fused_us"] = t_f
            log(f"[bench] low-bit gate/up with SwiGLU + quantiser fused {Mrows}x{F}x{K}: {t_f:.1f} us")
        del ws, q
    pr = out["projections"]
    out["per_layer_us"] = {"mxfp4": sum(v["mxfp4_us"] for v in pr.values()), "bf16": sum(v["bf16_us"] for v in pr.values())}
    return out


def bench_moe(B, g, Bn, N, w, steps, batches):
    """Decode steps of the paper's open-source mixture-of-experts recipe (random cache contents, fixed context)."""
    import torch
    from paper_2510_24824_amd import synth
    pos = N - 1
    # ---- the paper's open-source mixture-of-experts recipe: 16 layers, hidden 2048, 16 heads of 128, 64 SwiGLU
    # experts of hidden 1024 each, 8 per token (about 1B active / 7B total parameters)
    mo = {}
    mshape = synth.PLT_MOE_1B7B
    mblob = fill_weights_on_device(B, B.make_config(mshape, dtype=B.PLT_BF16), SEED + 4)
    for bn in batches:
        mtok = torch.randint(0, mshape.vocab, (bn,), generator=g, device="cuda", dtype=torch.int32)
        row = {}
        for name, mode, Lx in [("nonlooped_L1", B.PLT_MODE_CLP, 1), ("plt_L2", B.PLT_MODE_CLP, 2), ("plt_L3", B.PLT_MODE_CLP, 3),
                               ("vanilla_loop_L2", B.PLT_MODE_VANILLA_LOOP, 2)]:
            cm = B.make_config(mshape, dtype=B.PLT_BF16, mode=mode, n_loops=Lx, window=w)
            mm = B.Model(cm, mblob)
            km = B.KV(mm, bn, N)
            fill_kv_random(B, km, g)
            row[name] = time_steps(km, pos, mtok, 2, steps)
            km.close(); mm.close(); del km
            torch.cuda.empty_cache()
        row["latency_vs_nonlooped"] = {k: row[k] / row["nonlooped_L1"] for k in ("plt_L2", "plt_L3", "vanilla_loop_L2")}
        mo["batch_%d_ms_per_step" % bn] = row
        log(f"[bench] MoE 8-of-64 shape, batch {bn}: non-looped {row['nonlooped_L1']:.3f} ms, PLT-2 {row['plt_L2']:.3f}, "
            f"PLT-3 {row['plt_L3']:.3f}, vanilla loop 2 {row['vanilla_loop_L2']:.3f}")
    # the serving recipe on this shape: e4m3 caches + MXFP4 projections and experts (MXFP8 rows)
    lblob = fill_weights_on_device(B, B.make_config(mshape, dtype=B.PLT_BF16, w_dtype=B.PLT_MXFP4), SEED + 6)
    for bn in batches:
        mtok = torch.randint(0, mshape.vocab, (bn,), generator=g, device="cuda", dtype=torch.int32)
        row = {}
        for name, mode, Lx in [("nonlooped_L1", B.PLT_MODE_CLP, 1), ("plt_L2", B.PLT_MODE_CLP, 2), ("plt_L3", B.PLT_MODE_CLP, 3),
                               ("vanilla_loop_L2", B.PLT_MODE_VANILLA_LOOP, 2)]:
            cm = B.make_config(mshape, dtype=B.PLT_BF16, mode=mode, n_loops=Lx, window=w, kv_dtype=B.PLT_FP8_E4M3, w_dtype=B.PLT_MXFP4)
            mm = B.Model(cm, lblob)
            km = B.KV(mm, bn, N)
            fill_kv_random(B, km, g)
            row[name] = time_steps(km, pos, mtok, 2, steps)
            km.close(); mm.close(); del km
            torch.cuda.empty_cache()
        row["latency_vs_nonlooped"] = {k: row[k] / row["nonlooped_L1"] for k in ("plt_L2", "plt_L3", "vanilla_loop_L2")}
        row["tokens_per_s_plt_L2"] = bn / (row["plt_L2"] * 1e-3)
        mo["mxfp4_e4m3kv_batch_%d_ms_per_step" % bn] = row
        log(f"[bench] MoE shape, MXFP4 experts + e4m3 caches, batch {bn}: non-looped {row['nonlooped_L1']:.3f} ms, PLT-2 {row['plt_L2']:.3f}, "
            f"PLT-3 {row['plt_L3']:.3f}, vanilla loop 2 {row['vanilla_loop_L2']:.3f}")
    mo["mxfp4_weight_blob_bytes"] = int(lblob.numel()); mo["bf16_weight_blob_bytes"] = int(mblob.numel())
    del lblob
    mo["expert_weight_bytes_per_layer"] = 64 * 3 * mshape.ffn_hidden * mshape.d_model * 2
    mo["workload"] = ("16 layers, d=2048, 16 heads x 128, 64 SwiGLU experts of hidden 1024 (8 per row), vocab 50304, "
                      "%d-token context, bf16 caches" % N)
    del mblob
    torch.cuda.empty_cache()
    return mo


def measure_read_ceiling(B):
    """Practical HBM read ceiling on this machine: the library's plain read-only stream kernel over 4 GiB."""
    import torch
    src = torch.zeros(4 << 30, dtype=torch.uint8, device="cuda")
    out = torch.empty(4 << 20, dtype=torch.uint8, device="cuda")
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    call = lambda: B.lib().plt_stream_read(C.c_void_p(src.data_ptr()), src.numel(), C.c_void_p(out.data_ptr()), out.numel(), stream)
    for _ in range(3):
        assert call() == 0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        call()
    e1.record(); torch.cuda.synchronize()
    return src.numel() / (e0.elapsed_time(e1) * 1e-3 / 10) / 1e9


def read_traffic(name):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE), if a summary
    under profiles/ records it as a line `<name> = <bytes>`; else None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.strip().startswith(name) and "=" in line:
            try:
                return float(line.split("=", 1)[1].split()[0])
            except ValueError:
                return None
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--only-main", action="store_true", help="skip the baselines, the L sweep and the kernel-only run")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true", help="the full batch x context serving sweep (batch 1..256 x context 1024/2048/5000, 256 tokens, 5 runs: several minutes) instead of the reduced one")
    ap.add_argument("--no-sweep", action="store_true", help="skip the reduced serving sweep")
    ap.add_argument("--no-prefill", action="store_true", help="skip the CLP prefill of 4 x 8192 tokens at L=3 (configs[4])")
    ap.add_argument("--no-long-context", action="store_true",
                    help="skip the L=4, window 128, 8192-token configuration (configs[3]: batch 128 resident + parity, batch 256 aliased / e4m3)")
    ap.add_argument("--sweep-eager", action="store_true", help="serving sweep without the HIP-graph replay of the step")
    ap.add_argument("--attn-kernel-only", action="store_true", help="only the kernel-only fused attention configuration (bf16 and e4m3 caches)")
    ap.add_argument("--prefill-only", action="store_true", help="only the CLP prefill of 4 x 8192 tokens at L=3")
    ap.add_argument("--prefill-moe-only", action="store_true", help="only the CLP prefill of 4 x 8192 tokens at L=3 on the 8-of-64 mixture-of-experts shape")
    ap.add_argument("--copy-reference", action="store_true", help="only the plain copy kernel (reference for HBM traffic counters)")
    ap.add_argument("--sweep-moe", action="store_true", help="only the mixture-of-experts serving sweep (batch 4..64, context 5000, 256 tokens, 5 runs)")
    ap.add_argument("--moe-only", action="store_true", help="only the mixture-of-experts shape (8 of 64 experts) at batch 64")
    ap.add_argument("--lowbit-gemm-only", action="store_true", help="only the kernel-only low-bit (MXFP4 x MXFP8) GEMM comparison")
    ap.add_argument("--kv-fp8", action="store_true", help="main workload with e4m3 K/V caches (labelled variant)")
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--ctx", type=int, default=2048)
    ap.add_argument("--loops", type=int, default=2)
    ap.add_argument("--window", type=int, default=64)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_24824_amd import binding as B, synth
    B.lib()   # fails loudly if the HIP library is missing
    shape = synth.PLT_1P3B
    if args.copy_reference:
        print(json.dumps(copy_reference(B)), flush=True)
        return
    if args.attn_kernel_only:
        print(json.dumps({"attn_kernel_only": bench_attn_kernel(B, args.steps, args.warmup),
                          "attn_kernel_only_fp8_kv": bench_attn_kernel(B, args.steps, args.warmup, fp8=True)}), flush=True)
        return
    if args.sweep_moe:
        g0 = torch.Generator(device="cuda"); g0.manual_seed(SEED + 1)
        print(json.dumps({"serving_sweep_moe": bench_sweep_moe(B, g0)}), flush=True)
        return
    if args.moe_only:
        g0 = torch.Generator(device="cuda"); g0.manual_seed(SEED + 1)
        print(json.dumps({"moe_shape": bench_moe(B, g0, args.batch, args.ctx, args.window, max(8, args.steps // 2), (args.batch,))}), flush=True)
        return
    if args.lowbit_gemm_only:
        print(json.dumps({"lowbit_gemm": bench_lowbit_gemm(B, args.batch * args.loops)}), flush=True)
        return
    if args.prefill_moe_only:
        mshape = synth.PLT_MOE_1B7B
        cfg0 = B.make_config(mshape, dtype=B.PLT_BF16)
        g0 = torch.Generator(device="cuda"); g0.manual_seed(SEED + 1)
        print(json.dumps({"prefill_moe": bench_prefill(B, mshape, fill_weights_on_device(B, cfg0, SEED), g0)}), flush=True)
        return
    if args.prefill_only:
        cfg0 = B.make_config(shape, dtype=B.PLT_BF16)
        g0 = torch.Generator(device="cuda"); g0.manual_seed(SEED + 1)
        print(json.dumps({"prefill": bench_prefill(B, shape, fill_weights_on_device(B, cfg0, SEED), g0)}), flush=True)
        return
    kvd = B.PLT_FP8_E4M3 if args.kv_fp8 else 0
    Bn, N, L, w = args.batch, args.ctx, args.loops, args.window
    pos = N - 1                                  # the position a timed step consumes; it attends N keys

    cfg = B.make_config(shape, dtype=B.PLT_BF16, n_loops=L, window=w, kv_dtype=kvd)
    t0 = time.perf_counter()
    blob = fill_weights_on_device(B, cfg, SEED)
    model = B.Model(cfg, blob)
    kv = B.KV(model, Bn, N)
    g = torch.Generator(device="cuda"); g.manual_seed(SEED + 1)
    prompt = torch.randint(0, shape.vocab, (Bn, pos), generator=g, device="cuda", dtype=torch.int32)
    torch.cuda.synchronize()
    log(f"[bench] weights + KV allocated in {time.perf_counter() - t0:.1f} s; prefill of {Bn} x {pos} tokens ...")
    t0 = time.perf_counter()
    nxt, _ = kv.prefill(prompt, want_logits=False)
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0
    log(f"[bench] prefill done in {prefill_s:.2f} s")

    # state before the first decode step (for the oracle sample), then one clean step
    sample = sorted(set(int(round(i * (Bn - 1) / 5)) for i in range(6)))   # six sequences: 10-15 s of CPU work
    state = {}
    if not args.no_cpu_baseline:
        carry_all = kv.get_carry() if L > 1 else np.zeros((Bn, 0, shape.d_model), np.float32)
        for b in sample:
            state[b] = ([kv.export(b, m, pos) for m in range(shape.n_layers)], carry_all[b], int(nxt[b].item()))
    tok = nxt.clone()
    n1, lg1 = kv.decode_step(tok)
    hid1 = kv.get_hidden()
    gpu_logits = {b: lg1[b].float().cpu().numpy().astype(np.float64) for b in sample}
    gpu_hidden = {b: hid1[b].astype(np.float64) for b in sample}
    gpu_next = {b: int(n1[b].item()) for b in sample}

    # ---- timed region: K steps at fixed context; every attention launch bracketed by HIP events
    model.profile_enable(1 << B.PLT_PROF_ATTN)
    for _ in range(args.warmup):
        kv.set_position(pos); kv.decode_step(tok, want_logits=False)
    model.profile_read(B.PLT_PROF_ATTN, reset=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        kv.set_position(pos); kv.decode_step(tok, want_logits=False)
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps
    attn_ms, attn_n = model.profile_read(B.PLT_PROF_ATTN, reset=True)
    # second, separate pass: the GEMM launches bracketed instead (97 per step; kept out of `value`)
    model.profile_enable(1 << B.PLT_PROF_GEMM)
    time_steps(kv, pos, tok, 1, args.steps)
    gemm_ms, gemm_n = model.profile_read(B.PLT_PROF_GEMM, reset=True)
    model.profile_enable(0)
    ms_step_noevents = time_steps(kv, pos, tok, 2, args.steps)

    abytes = attn_alg_bytes(Bn, L, shape.n_heads, shape.n_kv_heads, shape.head_dim, N, w, 2, 1 if kvd else 2)
    attn_us = attn_ms * 1e3 / max(attn_n, 1)
    achieved = abytes / (attn_us * 1e-6) / 1e9
    wbytes = 2 * (shape.n_layers * ((shape.n_heads + 2 * shape.n_kv_heads) * shape.head_dim * shape.d_model
                                    + shape.d_model * shape.n_heads * shape.head_dim + 3 * shape.ffn_hidden * shape.d_model)
                  + shape.vocab * shape.d_model)
    out = {
        "metric": "decode tokens/s + step latency vs non-looped at L=2/3/4; attn HBM GB/s",
        "value": Bn / (ms_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 (e4m3 K/V caches)" if kvd else "bf16",
        "data": "synthetic",
        "config": {"workload": f"full CLP decode step, ~1.3B dense PLT (24 layers, d=2048, 16 heads x 128, SwiGLU 5632, vocab 32000), "
                               f"bf16{' with e4m3 K/V caches' if kvd else ''}, L={L}, window {w}, batch {Bn}, {N}-token shared KV context (configs[2])",
                   "batch": Bn, "n_loops": L, "window": w, "context": N, "seed": SEED,
                   "kv_fill": f"plt_prefill of {pos} uniform token ids per sequence ({prefill_s:.2f} s)"},
        "roofline": {"bound": "hbm", "kernel": f"k_attn_decode<128{', e4m3' if kvd else ''}> (fused decode attention, one launch per layer)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": read_traffic("attn_decode_c3_fp8kv_bytes_per_launch" if kvd else "attn_decode_c3_bytes_per_launch")
                     if (Bn, N, L, w) == (64, 2048, 2, 64) else None,
                     "algorithmic_bytes_per_launch": abytes, "avg_launch_us": attn_us, "launches": attn_n},
        "gemm": {"avg_launch_us": gemm_ms * 1e3 / max(gemm_n, 1), "launches": gemm_n,
                 "weight_bytes_per_step": wbytes, "ms_per_step": gemm_ms / args.steps,
                 "weight_GBps": wbytes / (gemm_ms / args.steps * 1e-3) / 1e9 if gemm_ms > 0 else None},
        "attn_ms_per_step": attn_ms / args.steps,
        "ms_per_step_without_event_instrumentation": ms_step_noevents,
        "kv_bytes_logical": model.kv_logical_bytes(Bn, N),
    }
    ceiling = measure_read_ceiling(B)
    out["roofline"]["measured_stream_read_GBps"] = ceiling          # context: what a plain read kernel reaches here
    out["roofline"]["frac_of_measured_stream_read"] = achieved / ceiling
    if not args.no_cpu_baseline:
        log(f"[bench] timing the CPU oracle on {len(sample)} sequences (10-15 s) ...")
        out["cpu_baseline"] = oracle_sample(B, shape, cfg, blob, state, pos, gpu_logits, gpu_hidden, gpu_next, kv=kv)
        log(f"[bench] parity: logits {out['cpu_baseline']['parity_max_abs_logits']:.2e}, per layer (teacher-forced) "
            f"{out['cpu_baseline']['parity_per_layer_teacher_forced_max_abs']:.2e}")
        state.clear()

    if not args.only_main and not kvd:
        # ---- same library, same weights: non-looped, the L sweep and the vanilla sequential loop.
        # Their caches are filled with N(0, 0.5) values on the device (timing only).
        kv.close(); del kv
        torch.cuda.empty_cache()
        lat = {}
        for name, mode, Lx in [("nonlooped_L1", B.PLT_MODE_CLP, 1), ("plt_L2", B.PLT_MODE_CLP, 2), ("plt_L3", B.PLT_MODE_CLP, 3),
                               ("plt_L4", B.PLT_MODE_CLP, 4), ("vanilla_loop_L2", B.PLT_MODE_VANILLA_LOOP, 2),
                               ("vanilla_loop_L3", B.PLT_MODE_VANILLA_LOOP, 3), ("vanilla_loop_L4", B.PLT_MODE_VANILLA_LOOP, 4),
                               # the paper's component table at L = 2: + CLP (per-loop KV), + KV share, + G-SWA (= plt_L2)
                               ("clp_own_kv_L2", B.PLT_MODE_CLP_OWN_KV, 2), ("clp_share_only_L2", B.PLT_MODE_CLP_SHARE_ONLY, 2)]:
            c2 = B.make_config(shape, dtype=B.PLT_BF16, mode=mode, n_loops=Lx, window=w)
            m2 = B.Model(c2, blob)
            k2 = B.KV(m2, Bn, N)
            fill_kv_random(B, k2, g)
            lat[name] = time_steps(k2, pos, tok, 2, max(8, args.steps // 2))
            log(f"[bench] {name}: {lat[name]:.3f} ms/step")
            k2.close(); m2.close(); del k2
            torch.cuda.empty_cache()
        base = lat["nonlooped_L1"]
        out["latency_ms"] = lat
        out["latency_vs_nonlooped"] = {k: v / base for k, v in lat.items()}
        out["component_table_L2"] = {"rows": ["(1) non-looped", "(2) + loop-2 (sequential, 2x KV)", "(3) + CLP (per-loop KV)",
                                              "(4) + KV share", "(5) + G-SWA = PLT-2"],
                                     "ms": [lat["nonlooped_L1"], lat["vanilla_loop_L2"], lat["clp_own_kv_L2"],
                                            lat["clp_share_only_L2"], lat["plt_L2"]]}
        out["attn_kernel_only"] = bench_attn_kernel(B, args.steps, args.warmup)
        # ---- the same step with e4m3 (FP8) K/V caches: the paper's serving setting, half the KV bytes.
        # Separate rows: `value` above is the bf16-cache number.
        f8 = {}
        for name, Lx in [("nonlooped_L1", 1), ("plt_L2", 2), ("plt_L3", 3), ("plt_L4", 4)]:
            c8 = B.make_config(shape, dtype=B.PLT_BF16, n_loops=Lx, window=w, kv_dtype=B.PLT_FP8_E4M3)
            m8 = B.Model(c8, blob)
            k8 = B.KV(m8, Bn, N)
            fill_kv_random(B, k8, g)
            m8.profile_enable(1 << B.PLT_PROF_ATTN)
            ms8 = time_steps(k8, pos, tok, 2, max(8, args.steps // 2))
            a_ms, a_n = m8.profile_read(B.PLT_PROF_ATTN, reset=True)
            ab8 = attn_alg_bytes(Bn, Lx, shape.n_heads, shape.n_kv_heads, shape.head_dim, N, w, 2, 1)
            us8 = a_ms * 1e3 / max(a_n, 1)
            f8[name] = {"ms_per_step": ms8, "tokens_per_s": Bn / (ms8 * 1e-3), "attn_us_per_launch": us8,
                        "attn_algorithmic_bytes": ab8, "attn_GBps": ab8 / (us8 * 1e-6) / 1e9,
                        "kv_bytes_logical": m8.kv_logical_bytes(Bn, N)}
            log(f"[bench] e4m3 caches {name}: {ms8:.3f} ms/step, attention {us8:.0f} us = {ab8 / (us8 * 1e-6) / 1e12:.2f} TB/s")
            k8.close(); m8.close(); del k8
            torch.cuda.empty_cache()
        f8["latency_vs_nonlooped"] = {k: f8[k]["ms_per_step"] / f8["nonlooped_L1"]["ms_per_step"] for k in ("plt_L2", "plt_L3", "plt_L4")}
        f8["attn_kernel_only"] = bench_attn_kernel(B, args.steps, args.warmup, fp8=True)
        out["fp8_kv_cache"] = f8
        # ---- the paper's open-source dense recipe: 16 layers, FFN 16384, 32 query / 8 kv heads of 64 (GQA)
        gq = {}
        gshape = synth.PLT_DENSE_GQA
        gblob = fill_weights_on_device(B, B.make_config(gshape, dtype=B.PLT_BF16), SEED + 3)
        gtok = torch.randint(0, gshape.vocab, (Bn,), generator=g, device="cuda", dtype=torch.int32)
        for name, mode, Lx in [("nonlooped_L1", B.PLT_MODE_CLP, 1), ("plt_L2", B.PLT_MODE_CLP, 2), ("plt_L3", B.PLT_MODE_CLP, 3),
                               ("vanilla_loop_L2", B.PLT_MODE_VANILLA_LOOP, 2)]:
            cg = B.make_config(gshape, dtype=B.PLT_BF16, mode=mode, n_loops=Lx, window=w)
            mg = B.Model(cg, gblob)
            kg = B.KV(mg, Bn, N)
            fill_kv_random(B, kg, g)
            mg.profile_enable(1 << B.PLT_PROF_ATTN)
            msg = time_steps(kg, pos, gtok, 2, max(8, args.steps // 2))
            a_ms, a_n = mg.profile_read(B.PLT_PROF_ATTN, reset=True)
            abg = attn_alg_bytes(Bn, Lx if mode == B.PLT_MODE_CLP else 1, gshape.n_heads, gshape.n_kv_heads, gshape.head_dim, N, w)
            usg = a_ms * 1e3 / max(a_n, 1)
            gq[name] = {"ms_per_step": msg, "tokens_per_s": Bn / (msg * 1e-3), "attn_us_per_launch": usg,
                        "attn_GBps": abg / (usg * 1e-6) / 1e9}
            log(f"[bench] dense GQA shape {name}: {msg:.3f} ms/step, attention {usg:.0f} us = {abg / (usg * 1e-6) / 1e12:.2f} TB/s")
            kg.close(); mg.close(); del kg
            torch.cuda.empty_cache()
        gq["latency_vs_nonlooped"] = {k: gq[k]["ms_per_step"] / gq["nonlooped_L1"]["ms_per_step"] for k in ("plt_L2", "plt_L3", "vanilla_loop_L2")}
        gq["workload"] = "16 layers, d=2048, FFN 16384, 32 query / 8 kv heads x 64, vocab 50304, batch %d, %d-token context" % (Bn, N)
        del gblob
        torch.cuda.empty_cache()
        out["dense_gqa_shape"] = gq
        out["moe_shape"] = bench_moe(B, g, Bn, N, w, max(8, args.steps // 2), (4, 16, Bn))
        out["lowbit_gemm"] = bench_lowbit_gemm(B, Bn * L)
        # ---- the serving recipe as a whole: e4m3 K/V caches + the four per-layer projections on MXFP4 weights /
        # MXFP8 activations (the reading taken for "FP8 self-attention and W4A8 linear layers"); same model shape
        lb = {}
        lcfg = B.make_config(shape, dtype=B.PLT_BF16, w_dtype=B.PLT_MXFP4)
        lblob = fill_weights_on_device(B, lcfg, SEED + 5)
        lb["weight_blob_bytes"] = int(lblob.numel()); lb["bf16_weight_blob_bytes"] = int(blob.numel())
        for name, Lx, kvd in [("nonlooped_L1_fp8kv", 1, B.PLT_FP8_E4M3), ("plt_L2_fp8kv", 2, B.PLT_FP8_E4M3),
                              ("plt_L3_fp8kv", 3, B.PLT_FP8_E4M3), ("plt_L2_bf16kv", 2, 0)]:
            cl = B.make_config(shape, dtype=B.PLT_BF16, n_loops=Lx, window=w, kv_dtype=kvd, w_dtype=B.PLT_MXFP4)
            ml = B.Model(cl, lblob)
            kl = B.KV(ml, Bn, N)
            fill_kv_random(B, kl, g)
            msl = time_steps(kl, pos, tok, 2, max(8, args.steps // 2))
            lb[name] = {"ms_per_step": msl, "tokens_per_s": Bn / (msl * 1e-3)}
            log(f"[bench] MXFP4 projections {name}: {msl:.3f} ms/step")
            kl.close(); ml.close(); del kl
            torch.cuda.empty_cache()
        lb["latency_vs_nonlooped"] = {k: lb[k]["ms_per_step"] / lb["nonlooped_L1_fp8kv"]["ms_per_step"] for k in ("plt_L2_fp8kv", "plt_L3_fp8kv")}
        del lblob
        torch.cuda.empty_cache()
        out["lowbit_model"] = lb

    if not args.only_main and not kvd:
        if args.sweep:
            out["serving_sweep"] = bench_sweep(B, shape, blob, g, graph=not args.sweep_eager)
        elif not args.no_sweep:
            # reduced form of the paper's serving protocol (256 tokens, mean of 5): 128 tokens, mean of 2, three batches x two contexts
            out["serving_sweep"] = bench_sweep(B, shape, blob, g, n_new=128, runs=2, contexts=(1024, 5000), batches=(1, 16, 64),
                                               graph=not args.sweep_eager)
            out["serving_sweep"]["note"] = "reduced: 128 decoded tokens, mean of 2 runs; --sweep runs the full protocol"
        if not args.no_prefill:
            out["prefill"] = bench_prefill(B, shape, blob, g)
            log(f"[bench] prefill 4 x 8192, L=3: {out['prefill']['ms']:.0f} ms, {out['prefill']['roofline']['achieved']:.0f} TFLOP/s")
        if not args.no_long_context:
            out["long_context"] = bench_long_context(B, shape, blob, g, max(4, args.steps // 4), parity=not args.no_cpu_baseline)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
