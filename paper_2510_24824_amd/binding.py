"""Thin ctypes binding of libplt.so: same names as include/plt.h, argument marshalling only.

torch is used for device memory and the current stream; every step of the path runs in the
library's HIP kernels.  There is no CPU fallback: a missing library raises at load time.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libplt.so")

PLT_F32, PLT_BF16 = 0, 1
PLT_FP8_E4M3 = 2      # cache-only element type (e4m3 bytes); q / y / weights stay bf16
PLT_MXFP4 = 3         # weight-only element type of the low-bit projections
PLT_MODE_CLP, PLT_MODE_VANILLA_LOOP, PLT_MODE_CLP_SHARE_ONLY, PLT_MODE_CLP_OWN_KV = 0, 2, 3, 4
(PLT_W_EMB, PLT_W_NORM1, PLT_W_WQKV, PLT_W_GATE_W, PLT_W_GATE_B, PLT_W_WO, PLT_W_NORM2, PLT_W_WGU,
 PLT_W_WDOWN, PLT_W_NORM_F, PLT_W_HEAD, PLT_W_ROUTER, PLT_W_WQKV_SC, PLT_W_WO_SC, PLT_W_WGU_SC,
 PLT_W_WDOWN_SC) = range(16)
STATUS = {0: "PLT_OK", -1: "PLT_EINVAL", -2: "PLT_ENOMEM", -3: "PLT_ECTXFULL", -4: "PLT_EHIP", -5: "PLT_ESTATE"}


class PltError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{STATUS.get(code, code)}: {msg}")
        self.code = code


class plt_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "head_dim",
                                         "ffn_hidden", "vocab", "n_loops", "window", "dtype", "mode",
                                         "tie_embeddings")] + [("rope_theta", C.c_float), ("norm_eps", C.c_float),
                                                               ("kv_dtype", C.c_int32), ("n_experts", C.c_int32),
                                                               ("top_k", C.c_int32), ("w_dtype", C.c_int32)]


_P, _I, _Z = C.c_void_p, C.c_int32, C.c_size_t
_SIGS = {
    "plt_weights_bytes": (_Z, [C.POINTER(plt_config)]),
    "plt_weights_offset": (C.c_int, [C.POINTER(plt_config), _I, _I, C.POINTER(_Z), C.POINTER(_Z)]),
    "plt_init": (C.c_int, [C.POINTER(plt_config), _P, _Z, _P, C.POINTER(_P)]),
    "plt_free": (None, [_P]),
    "plt_kv_bytes": (_Z, [_P, _I, _I]),
    "plt_kv_logical_bytes": (_Z, [_P, _I, _I]),
    "plt_kv_alloc": (C.c_int, [_P, _I, _I, _P, _Z, C.POINTER(_P)]),
    "plt_kv_free": (None, [_P]),
    "plt_prefill_workspace_bytes": (_Z, [_P, _P, _I]),
    "plt_prefill": (C.c_int, [_P, _P, _P, _I, _P, _P, _P, _Z]),
    "plt_decode_step": (C.c_int, [_P, _P, _P, _P, _P]),
    "plt_kv_alias_layers": (C.c_int, [_P, _I]),
    "plt_use_graph": (C.c_int, [_P, _I]),
    "plt_kv_position": (_I, [_P]),
    "plt_last_error": (C.c_char_p, []),
    "plt_kv_set_position": (C.c_int, [_P, _I]),
    "plt_kv_export_bytes": (_Z, [_P, _I]),
    "plt_kv_export": (C.c_int, [_P, _I, _I, _I, _I, _P, _Z]),
    "plt_kv_import": (C.c_int, [_P, _I, _I, _I, _I, _P, _Z]),
    "plt_get_carry": (C.c_int, [_P, _P, _Z]),
    "plt_set_carry": (C.c_int, [_P, _P, _Z]),
    "plt_get_hidden": (C.c_int, [_P, _P, _Z]),
    "plt_debug_layer": (C.c_int, [_P, _P, _I, _P, _P, _Z]),
    "plt_debug_act_codes": (C.c_int, [_P, _I, _P, _Z, _P, _Z]),
    "plt_attn_pad32": (_I, [_I]),
    "plt_attn_pad": (_I, [_I, _I]),
    "plt_attn_scratch_bytes": (_Z, [_I, _I, _I, _I, _I]),
    "plt_attn_decode": (C.c_int, [_I] * 10 + [_P] * 8 + [_Z, _I, _P]),
    "plt_attn_decode_static": (C.c_int, [_I] * 10 + [_P] * 7 + [_I, _P]),
    "plt_attn_k_index": (C.c_int64, [_I, _I, _I, _I]),
    "plt_attn_v_index": (C.c_int64, [_I, _I, _I, _I]),
    "plt_attn_pack_k": (C.c_int, [_I, _I, _I, _I, _P, _P, _P]),
    "plt_attn_pack_v": (C.c_int, [_I, _I, _I, _I, _P, _P, _P]),
    "plt_gemm": (C.c_int, [_I, _I, _I, _I, _P, _P, _P, _P, _Z, _P]),
    "plt_gemm_scratch_bytes": (_Z, [_I, _I, _I]),
    "plt_gemm_residual": (C.c_int, [_I, _I, _I, _P, _P, _P, _P]),
    "plt_moe_weight_index": (C.c_int64, [_I, _I, _I]),
    "plt_moe_scratch_bytes": (_Z, [_I] * 6),
    "plt_moe_ffn": (C.c_int, [_I] * 6 + [_P] * 8 + [_Z, _P]),
    "plt_mx_weight_code_bytes": (_Z, [_I, _I]),
    "plt_mx_weight_scale_bytes": (_Z, [_I, _I]),
    "plt_mx_act_scale_bytes": (_Z, [_I, _I]),
    "plt_mx_weight_code_index": (C.c_int64, [_I, _I, _I]),
    "plt_mx_weight_scale_index": (C.c_int64, [_I, _I, _I]),
    "plt_mx_act_scale_index": (_I, [_I]),
    "plt_mx_quantize_weights": (C.c_int, [_I, _I, _P, _P, _P, _P]),
    "plt_mx_quantize_act": (C.c_int, [_I, _I, _I, _P, _P, _P, _P]),
    "plt_gemm_mx_scratch_bytes": (_Z, [_I, _I, _I]),
    "plt_gemm_mx": (C.c_int, [_I, _I, _I, _P, _P, _P, _P, _P, _P, _Z, _P]),
    "plt_gemm_mx_swiglu_scratch_bytes": (_Z, [_I, _I, _I]),
    "plt_gemm_mx_swiglu": (C.c_int, [_I, _I, _I, _P, _P, _P, _P, _P, _P, _P, _Z, _P]),
    "plt_stream_copy": (C.c_int, [_P, _P, _Z, _P]),
    "plt_stream_read": (C.c_int, [_P, _Z, _P, _Z, _P]),
    "plt_profile_enable": (C.c_int, [_P, _I]),
    "plt_profile_read": (C.c_int, [_P, _I, C.POINTER(C.c_double), C.POINTER(C.c_int64), _I]),
}
PLT_PROF_ATTN, PLT_PROF_GEMM = 0, 1
EXPORTS = tuple(_SIGS)

_lib = None


def lib():
    """Loads libplt.so (built by paper_2510_24824_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not found: build it with __graft_entry__.build() "
                                    "(python -m paper_2510_24824_amd.build); there is no fallback path")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def _check(rc):
    if rc != 0:
        raise PltError(rc, lib().plt_last_error().decode())


def make_config(shape, dtype=PLT_BF16, mode=PLT_MODE_CLP, n_loops=None, window=None, kv_dtype=0, w_dtype=0) -> plt_config:
    return plt_config(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.head_dim,
                      shape.ffn_hidden, shape.vocab, shape.n_loops if n_loops is None else n_loops,
                      shape.window if window is None else window, dtype, mode,
                      1 if shape.tie_embeddings else 0, shape.rope_theta, shape.norm_eps, kv_dtype,
                      getattr(shape, "n_experts", 0), getattr(shape, "top_k", 0), w_dtype)


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def weights_offset(cfg, layer, which):
    off, n = _Z(), _Z()
    _check(lib().plt_weights_offset(C.byref(cfg), layer, which, C.byref(off), C.byref(n)))
    return off.value, n.value


def moe_tile_weights(w: np.ndarray) -> np.ndarray:
    """Expert matrices [..., N, K] (N % 16 == 0, K % 32 == 0) -> the strip order of the bf16 blob:
    [..., strip, k chunk, k/8 mod 4, n mod 16, k mod 8] (see plt_moe_weight_index); a pure permutation."""
    *lead, N, K = w.shape
    assert N % 16 == 0 and K % 32 == 0, (N, K)
    t = w.reshape(*lead, N // 16, 16, K // 32, 4, 8)
    nl = len(lead)
    t = np.transpose(t, tuple(range(nl)) + (nl, nl + 2, nl + 3, nl + 1, nl + 4))
    return np.ascontiguousarray(t).reshape(*lead, N, K)


def pack_weights(cfg: plt_config, weights: dict, device="cuda"):
    """Copies a weight dict (float32 arrays, [out, in]) into a device blob in the library's layout."""
    import torch
    from . import synth
    nbytes = lib().plt_weights_bytes(C.byref(cfg))
    if nbytes == 0:
        raise PltError(-1, lib().plt_last_error().decode())
    host = np.zeros(nbytes, np.uint8)

    def put(layer, which, arr, model_dtype):
        off, n = weights_offset(cfg, layer, which)
        arr = np.ascontiguousarray(arr, np.float32).reshape(-1)
        assert arr.size == n, (which, arr.size, n)
        if model_dtype and cfg.dtype == PLT_BF16:
            host[off:off + 2 * n] = synth.bf16_bits(arr).view(np.uint8)
        else:
            host[off:off + 4 * n] = arr.view(np.uint8)

    mx = cfg.w_dtype == PLT_MXFP4
    later = []          # low-bit projections: quantised on the device, straight into the blob

    def put_w(layer, which, which_sc, arr):
        if mx:
            later.append((layer, which, which_sc, np.ascontiguousarray(arr, np.float32), 0))
        else:
            put(layer, which, arr, True)

    put(0, PLT_W_EMB, weights["emb"], True)
    for m, lw in enumerate(weights["layers"]):
        put(m, PLT_W_NORM1, lw["norm1"], False)
        put_w(m, PLT_W_WQKV, PLT_W_WQKV_SC, np.concatenate([lw["wq"], lw["wk"], lw["wv"]], axis=0))
        put(m, PLT_W_GATE_W, lw["gate_w"], False)
        put(m, PLT_W_GATE_B, lw["gate_b"], False)
        put_w(m, PLT_W_WO, PLT_W_WO_SC, lw["wo"])
        put(m, PLT_W_NORM2, lw["norm2"], False)
        if cfg.n_experts > 0 and mx:     # every expert's matrices quantised one by one
            put(m, PLT_W_ROUTER, lw["router"], True)
            gu = np.concatenate([lw["w_gate"], lw["w_up"]], axis=1)
            for e in range(cfg.n_experts):
                later.append((m, PLT_W_WGU, PLT_W_WGU_SC, np.ascontiguousarray(gu[e], np.float32), e))
                later.append((m, PLT_W_WDOWN, PLT_W_WDOWN_SC, np.ascontiguousarray(lw["w_down"][e], np.float32), e))
        elif cfg.n_experts > 0:       # expert axis first; per expert its gate rows, then its up rows
            tile = moe_tile_weights if cfg.dtype == PLT_BF16 else (lambda x: x)
            put(m, PLT_W_ROUTER, lw["router"], True)
            put(m, PLT_W_WGU, tile(np.concatenate([lw["w_gate"], lw["w_up"]], axis=1)), True)
            put(m, PLT_W_WDOWN, tile(np.asarray(lw["w_down"])), True)
        else:
            put_w(m, PLT_W_WGU, PLT_W_WGU_SC, np.concatenate([lw["w_gate"], lw["w_up"]], axis=0))
            put_w(m, PLT_W_WDOWN, PLT_W_WDOWN_SC, lw["w_down"])
    put(0, PLT_W_NORM_F, weights["norm_f"], False)
    if not cfg.tie_embeddings:
        put(0, PLT_W_HEAD, weights["head"], True)
    blob = torch.from_numpy(host).to(device)
    for layer, which, which_sc, arr, index in later:
        quantize_into_blob(cfg, blob, layer, which, which_sc, torch.from_numpy(arr).to(device).to(torch.bfloat16), index)
    return blob


def quantize_into_blob(cfg, blob, layer, which, which_sc, w_bf16, index=0):
    """Low-bit models: quantises one bf16 projection matrix [N, K] (device) into its two blob tensors
    (index: which of the tensor's back-to-back matrices, i.e. the expert)."""
    N, K = w_bf16.shape
    off, n = weights_offset(cfg, layer, which)
    off_sc, n_sc = weights_offset(cfg, layer, which_sc)
    sb = lib().plt_mx_weight_scale_bytes(N, K)
    count = max(cfg.n_experts, 1) if which in (PLT_W_WGU, PLT_W_WDOWN) else 1
    assert n == count * N * K and n_sc == count * sb and index < count, (which, n, N, K)
    _check(lib().plt_mx_quantize_weights(N, K, _ptr(w_bf16.contiguous()), C.c_void_p(blob.data_ptr() + off + index * (N * K // 2)),
                                         C.c_void_p(blob.data_ptr() + off_sc + index * sb), _stream()))


class Model:
    """plt_model + its weight blob (kept alive here)."""

    def __init__(self, cfg: plt_config, blob):
        self.cfg, self.blob = cfg, blob
        h = _P()
        _check(lib().plt_init(C.byref(cfg), _ptr(blob), blob.numel(), _stream(), C.byref(h)))
        self.h = h

    def kv_bytes(self, batch, max_ctx):
        return lib().plt_kv_bytes(self.h, batch, max_ctx)

    def kv_logical_bytes(self, batch, n_ctx):
        return lib().plt_kv_logical_bytes(self.h, batch, n_ctx)

    def kv_alias_layers(self, phys_layers):
        """Timing only: kv objects created afterwards keep `phys_layers` layers of shared cache (0: all)."""
        _check(lib().plt_kv_alias_layers(self.h, int(phys_layers)))

    def use_graph(self, on=True):
        """plt_decode_step replays its launch sequence as one HIP graph (captured on first use)."""
        _check(lib().plt_use_graph(self.h, 1 if on else 0))

    def profile_enable(self, mask):
        """mask: OR of (1 << PLT_PROF_ATTN), (1 << PLT_PROF_GEMM); 0 switches the instrumentation off."""
        _check(lib().plt_profile_enable(self.h, int(mask)))

    def profile_read(self, klass, reset=True):
        """(summed milliseconds, launches) of one kernel class since the last reset."""
        ms, cnt = C.c_double(), C.c_int64()
        _check(lib().plt_profile_read(self.h, klass, C.byref(ms), C.byref(cnt), 1 if reset else 0))
        return ms.value, cnt.value

    def close(self):
        if self.h:
            lib().plt_free(self.h)
            self.h = None


class KV:
    """plt_kv bound to a torch-owned device buffer."""

    def __init__(self, model: Model, batch: int, max_ctx: int):
        import torch
        self.model, self.batch, self.max_ctx = model, batch, max_ctx
        nbytes = model.kv_bytes(batch, max_ctx)
        if nbytes == 0:
            raise PltError(-1, lib().plt_last_error().decode())
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        h = _P()
        _check(lib().plt_kv_alloc(model.h, batch, max_ctx, _ptr(self.buf), nbytes, C.byref(h)))
        self.h = h
        self.next = torch.empty(batch, dtype=torch.int32, device="cuda")
        self.logits = torch.empty(batch, model.cfg.vocab, dtype=torch.float32, device="cuda")
        self._ws = None

    def prefill(self, tokens, want_logits=True):
        """tokens: int32 device tensor [batch, n]; returns (next ids, logits) device tensors."""
        assert tokens.dtype.is_floating_point is False and tokens.is_cuda and tokens.dim() == 2
        assert tokens.shape[0] == self.batch
        import torch
        tokens = tokens.contiguous()
        n = tokens.shape[1]
        nb = lib().plt_prefill_workspace_bytes(self.model.h, self.h, n)
        if nb == 0:       # an invalid prompt length: the call itself reports the precise status
            _check(lib().plt_prefill(self.model.h, self.h, _ptr(tokens), n, _ptr(self.next), None, None, 0))
            raise PltError(-1, "plt_prefill_workspace_bytes returned 0")
        # the workspace is the caller's: a torch buffer, kept until the kv object goes (the call is asynchronous)
        if self._ws is None or self._ws.numel() < nb:
            self._ws = None
            self._ws = torch.empty(nb, dtype=torch.uint8, device="cuda")
        _check(lib().plt_prefill(self.model.h, self.h, _ptr(tokens), n, _ptr(self.next),
                                 _ptr(self.logits) if want_logits else None, _ptr(self._ws), self._ws.numel()))
        return self.next, (self.logits if want_logits else None)

    def drop_workspace(self):
        """Frees the prefill workspace (after a synchronisation: the prefill that used it may still be running)."""
        import torch
        torch.cuda.synchronize()
        self._ws = None

    def decode_step(self, tokens, want_logits=True):
        tokens = tokens.contiguous()
        assert tokens.numel() == self.batch and tokens.is_cuda
        _check(lib().plt_decode_step(self.model.h, self.h, _ptr(tokens), _ptr(self.next),
                                     _ptr(self.logits) if want_logits else None))
        return self.next, (self.logits if want_logits else None)

    @property
    def position(self):
        return lib().plt_kv_position(self.h)

    def set_position(self, pos):
        _check(lib().plt_kv_set_position(self.h, pos))

    def _np_dtype(self):
        if self.model.cfg.kv_dtype == PLT_FP8_E4M3:
            return np.uint8
        return np.uint16 if self.model.cfg.dtype == PLT_BF16 else np.float32

    def export(self, seq, layer, n, cache=0):
        """Returns dict of float32 arrays: k_share, v_share [Hkv,n,D], k_ring, v_ring [L-1,Hkv,w,D]."""
        from . import synth
        c = self.model.cfg
        nbytes = lib().plt_kv_export_bytes(self.h, n)
        host = np.zeros(nbytes // np.dtype(self._np_dtype()).itemsize, self._np_dtype())
        _check(lib().plt_kv_export(self.h, seq, layer, cache, n, host.ctypes.data_as(_P), nbytes))
        vals = (synth.e4m3_from_bits(host) if c.kv_dtype == PLT_FP8_E4M3 else
                synth.bf16_from_bits(host) if c.dtype == PLT_BF16 else host)
        Hkv, D, w = c.n_kv_heads, c.head_dim, max(c.window, 1)
        nr = c.n_loops - 1 if c.mode == PLT_MODE_CLP else 0
        a = Hkv * n * D
        out = {"k_share": vals[:a].reshape(Hkv, n, D), "v_share": vals[a:2 * a].reshape(Hkv, n, D)}
        r = nr * Hkv * w * D
        out["k_ring"] = vals[2 * a:2 * a + r].reshape(nr, Hkv, w, D)
        out["v_ring"] = vals[2 * a + r:2 * a + 2 * r].reshape(nr, Hkv, w, D)
        return out

    def import_(self, seq, layer, n, k_share, v_share, k_ring=None, v_ring=None, cache=0):
        from . import synth
        c = self.model.cfg
        parts = [k_share, v_share] + ([k_ring, v_ring] if k_ring is not None else [])
        flat = np.concatenate([np.ascontiguousarray(p, np.float32).reshape(-1) for p in parts])
        host = (synth.e4m3_bits(flat) if c.kv_dtype == PLT_FP8_E4M3 else
                synth.bf16_bits(flat) if c.dtype == PLT_BF16 else flat)
        _check(lib().plt_kv_import(self.h, seq, layer, cache, n, host.ctypes.data_as(_P), host.nbytes))

    def get_carry(self):
        c = self.model.cfg
        out = np.zeros((self.batch, c.n_loops - 1, c.d_model), np.float32)
        _check(lib().plt_get_carry(self.h, out.ctypes.data_as(_P), out.nbytes))
        return out

    def set_carry(self, carry):
        carry = np.ascontiguousarray(carry, np.float32)
        _check(lib().plt_set_carry(self.h, carry.ctypes.data_as(_P), carry.nbytes))

    def get_hidden(self):
        c = self.model.cfg
        rows = 1 if c.mode == PLT_MODE_VANILLA_LOOP else c.n_loops
        out = np.zeros((self.batch, rows, c.d_model), np.float32)
        _check(lib().plt_get_hidden(self.h, out.ctypes.data_as(_P), out.nbytes))
        return out

    def debug_layer(self, layer, x_in):
        """One layer of block f on the decode micro-batch from a given residual stream x_in [batch, rows, d]
        (float32 numpy) at the position the next decode step would consume; returns the layer's output rows."""
        x_in = np.ascontiguousarray(x_in, np.float32)
        out = np.zeros_like(x_in)
        _check(lib().plt_debug_layer(self.model.h, self.h, layer, x_in.ctypes.data_as(_P), out.ctypes.data_as(_P), x_in.nbytes))
        return out

    def debug_act_codes(self, which):
        """Low-bit dense models: (e4m3 code bytes [rows, K], scale bytes [rows, 16 * ceil(K / 512)]) of the input of
        projection `which` (0 QKV, 1 output, 2 gate/up, 3 down) of the layer the last debug_layer call ran."""
        c = self.model.cfg
        K = c.n_heads * c.head_dim if which == 1 else (c.ffn_hidden if which == 3 else c.d_model)
        rows = self.batch * c.n_loops
        codes = np.zeros((rows, K), np.uint8)
        scales = np.zeros((rows, 16 * ((K + 511) // 512)), np.uint8)
        _check(lib().plt_debug_act_codes(self.h, which, codes.ctypes.data_as(_P), codes.nbytes, scales.ctypes.data_as(_P), scales.nbytes))
        return codes, scales

    def close(self):
        if self.h:
            import torch
            torch.cuda.synchronize()       # the workspace and the buffer go back to torch's allocator below
            lib().plt_kv_free(self.h)
            self.h = None
            self._ws = None


# ---- kernel-only hooks -------------------------------------------------------------------

def _to_dev(arr, dtype):
    """float32 numpy (exactly representable in the storage type) -> device tensor of the storage type
    (e4m3: a uint8 tensor of codes)."""
    import torch
    if dtype == PLT_FP8_E4M3:
        from . import synth
        return torch.from_numpy(synth.e4m3_bits(np.ascontiguousarray(arr, np.float32))).cuda()
    t = torch.from_numpy(np.ascontiguousarray(arr, np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == PLT_BF16 else t


def attn_pack_k(dtype, src, n):
    """src: device tensor [S, n, D] -> K layout [S, pad(n), D]."""
    import torch
    S, _, D = src.shape
    dst = torch.empty(S, lib().plt_attn_pad(dtype, n), D, dtype=src.dtype, device="cuda")
    _check(lib().plt_attn_pack_k(dtype, S, n, D, _ptr(src.contiguous()), _ptr(dst), _stream()))
    return dst


def attn_pack_v(dtype, src, n):
    """src: device tensor [S, n, D] -> the cache's V layout [S, pad(n) * D] (blocks of 32 positions in 16-byte chunks)."""
    import torch
    S, _, D = src.shape
    npad = lib().plt_attn_pad(dtype, n)
    dst = torch.empty(S, npad // 32, D, 32, dtype=src.dtype, device="cuda")
    _check(lib().plt_attn_pack_v(dtype, S, n, D, _ptr(src.contiguous()), _ptr(dst), _stream()))
    return dst


class AttnDecode:
    """Device-resident inputs of the kernel-only fused decode attention, in the native layout."""

    def __init__(self, dtype, q, k_share, v_share, k_ring, v_ring, z):
        import torch
        self.dtype = dtype
        B, L, Hq, D = q.shape
        Hkv, N = k_share.shape[1], k_share.shape[2]
        w = k_ring.shape[3] if L > 1 else 1
        self.dims = (B, L, Hq, Hkv, D, N, w)
        self.q = _to_dev(q, PLT_BF16 if dtype == PLT_FP8_E4M3 else dtype)
        self.ks = attn_pack_k(dtype, _to_dev(k_share, dtype).reshape(B * Hkv, N, D), N)
        self.vs = attn_pack_v(dtype, _to_dev(v_share, dtype).reshape(B * Hkv, N, D), N)
        if L > 1:
            self.kr = attn_pack_k(dtype, _to_dev(k_ring, dtype).reshape(B * (L - 1) * Hkv, w, D), w)
            self.vr = attn_pack_v(dtype, _to_dev(v_ring, dtype).reshape(B * (L - 1) * Hkv, w, D), w)
            self.z = torch.from_numpy(np.ascontiguousarray(z, np.float32)).cuda()
        else:
            self.kr = self.vr = self.z = None
        self.y = torch.empty_like(self.q)
        nb = lib().plt_attn_scratch_bytes(B, L, Hq, Hkv, D)
        self.scratch = torch.zeros(nb, dtype=torch.uint8, device="cuda")   # zero once; the library keeps it clean

    def run(self, n_ctx=None, n_ring=None, n_splits=0):
        B, L, Hq, Hkv, D, N, w = self.dims
        n_ctx = N if n_ctx is None else n_ctx
        n_ring = (w if n_ring is None else n_ring) if L > 1 else 0
        _check(lib().plt_attn_decode(self.dtype, B, L, Hq, Hkv, D, N, n_ctx, w, n_ring, _ptr(self.q), _ptr(self.ks),
                                     _ptr(self.vs), _ptr(self.kr), _ptr(self.vr), _ptr(self.z), _ptr(self.y),
                                     _ptr(self.scratch), self.scratch.numel(), n_splits, _stream()))
        return self.y

    def run_static(self, n_ctx=None, n_ring=None, n_splits=0, y=None):
        """The same call through the entry point that allocates nothing (split partials in the library's own
        device array); writes into y (default: a second output tensor kept by this object)."""
        import torch
        B, L, Hq, Hkv, D, N, w = self.dims
        n_ctx = N if n_ctx is None else n_ctx
        n_ring = (w if n_ring is None else n_ring) if L > 1 else 0
        if y is None:
            if getattr(self, "y_static", None) is None:
                self.y_static = torch.empty_like(self.q)
            y = self.y_static
        _check(lib().plt_attn_decode_static(self.dtype, B, L, Hq, Hkv, D, N, n_ctx, w, n_ring, _ptr(self.q), _ptr(self.ks),
                                            _ptr(self.vs), _ptr(self.kr), _ptr(self.vr), _ptr(self.z), _ptr(y), n_splits,
                                            _stream()))
        return y


def gemm(dtype, a, w):
    """a [M,K], w [N,K] device tensors of the storage type -> float32 [M,N]."""
    import torch
    M, K = a.shape
    N = w.shape[0]
    c = torch.empty(M, N, dtype=torch.float32, device="cuda")
    nb = lib().plt_gemm_scratch_bytes(M, N, K)
    scratch = torch.empty(nb, dtype=torch.uint8, device="cuda")
    _check(lib().plt_gemm(dtype, M, N, K, _ptr(a.contiguous()), _ptr(w.contiguous()), _ptr(c), _ptr(scratch), nb, _stream()))
    return c


def gemm_residual(a, w, x):
    """x [M,N] float32 (device, updated in place) += a [M,K] w [N,K]^T, bf16 device tensors, through the prefill tile kernel."""
    M, K = a.shape
    _check(lib().plt_gemm_residual(M, w.shape[0], K, _ptr(a.contiguous()), _ptr(w.contiguous()), _ptr(x), _stream()))
    return x


def moe_ffn(dtype, a, router, w_gate, w_up, w_down, top_k):
    """Kernel-only mixture-of-experts feed-forward.  a [R, d], router [E, d], w_gate / w_up [E, F, d],
    w_down [E, d, F]: float32 numpy arrays exactly representable in the storage type.  Returns
    (y [R, d] float32, sel_e [R, k] int32, sel_p [R, k] float32) as numpy arrays."""
    import torch
    R, d = a.shape
    E, F = w_gate.shape[0], w_gate.shape[1]
    tile = moe_tile_weights if dtype == PLT_BF16 else (lambda x: x)
    da, dr, dd = _to_dev(a, dtype), _to_dev(router, dtype), _to_dev(tile(np.asarray(w_down)), dtype)
    dgu = _to_dev(tile(np.concatenate([w_gate, w_up], axis=1)), dtype)
    y = torch.empty(R, d, dtype=torch.float32, device="cuda")
    sel_e = torch.empty(R, top_k, dtype=torch.int32, device="cuda")
    sel_p = torch.empty(R, top_k, dtype=torch.float32, device="cuda")
    nb = lib().plt_moe_scratch_bytes(dtype, R, d, F, E, top_k)
    if nb == 0:
        raise PltError(-1, lib().plt_last_error().decode())
    scratch = torch.empty(nb, dtype=torch.uint8, device="cuda")
    _check(lib().plt_moe_ffn(dtype, R, d, F, E, top_k, _ptr(da), _ptr(dr), _ptr(dgu), _ptr(dd), _ptr(y), _ptr(sel_e),
                             _ptr(sel_p), _ptr(scratch), nb, _stream()))
    torch.cuda.synchronize()
    return y.cpu().numpy(), sel_e.cpu().numpy(), sel_p.cpu().numpy()


# ---- low-bit (microscaling) projections ----------------------------------------------------

def mx_quantize_weights(w):
    """w: bf16 device tensor [N, K] -> (e2m1 codes, e8m0 scales) uint8 device tensors in the GEMM's layout."""
    import torch
    N, K = w.shape
    nc, ns = lib().plt_mx_weight_code_bytes(N, K), lib().plt_mx_weight_scale_bytes(N, K)
    if nc == 0 or ns == 0:
        raise PltError(-1, lib().plt_last_error().decode())
    codes = torch.empty(nc, dtype=torch.uint8, device="cuda")
    scales = torch.empty(ns, dtype=torch.uint8, device="cuda")
    _check(lib().plt_mx_quantize_weights(N, K, _ptr(w.contiguous()), _ptr(codes), _ptr(scales), _stream()))
    return codes, scales


def mx_quantize_act(x):
    """x: float32 or bf16 device tensor [M, K] -> (e4m3 codes [M, K], e8m0 scales [M, 16 * ceil(K / 512)])."""
    import torch
    M, K = x.shape
    ns = lib().plt_mx_act_scale_bytes(M, K)
    if ns == 0:
        raise PltError(-1, lib().plt_last_error().decode())
    codes = torch.empty(M, K, dtype=torch.uint8, device="cuda")
    scales = torch.empty(M, ns // M, dtype=torch.uint8, device="cuda")
    dt = PLT_F32 if x.dtype == torch.float32 else PLT_BF16
    _check(lib().plt_mx_quantize_act(dt, M, K, _ptr(x.contiguous()), _ptr(codes), _ptr(scales), _stream()))
    return codes, scales


def gemm_mx(a_codes, a_scales, w_codes, w_scales, M, N, K):
    """float32 [M, N] = dequantised a [M, K] times dequantised w [N, K]^T on the block-scaled matrix cores."""
    import torch
    c = torch.empty(M, N, dtype=torch.float32, device="cuda")
    nb = lib().plt_gemm_mx_scratch_bytes(M, N, K)
    if nb == 0:
        raise PltError(-1, lib().plt_last_error().decode())
    scratch = torch.empty(nb, dtype=torch.uint8, device="cuda")
    _check(lib().plt_gemm_mx(M, N, K, _ptr(a_codes), _ptr(a_scales), _ptr(w_codes), _ptr(w_scales), _ptr(c), _ptr(scratch), nb,
                             _stream()))
    return c


def gemm_mx_swiglu(a_codes, a_scales, w_codes, w_scales, M, F, K):
    """Low-bit gate/up projection + SwiGLU + block quantiser: (e4m3 codes [M, F], e8m0 scales [M, 16 * ceil(F / 512)])."""
    import torch
    nb = lib().plt_gemm_mx_swiglu_scratch_bytes(M, F, K)
    ns = lib().plt_mx_act_scale_bytes(M, F)
    if nb == 0 or ns == 0:
        raise PltError(-1, lib().plt_last_error().decode())
    codes = torch.empty(M, F, dtype=torch.uint8, device="cuda")
    scales = torch.empty(M, ns // M, dtype=torch.uint8, device="cuda")
    scratch = torch.empty(nb, dtype=torch.uint8, device="cuda")
    _check(lib().plt_gemm_mx_swiglu(M, F, K, _ptr(a_codes), _ptr(a_scales), _ptr(w_codes), _ptr(w_scales), _ptr(codes), _ptr(scales),
                                    _ptr(scratch), nb, _stream()))
    return codes, scales
