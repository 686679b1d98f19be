"""The entry point that allocates nothing (plt_attn_decode_static: split partials in a device array the library
itself holds) against the existing entry point plt_attn_decode on the same inputs: identical bits, on two calls in a
row, the second with a smaller input; a shape whose partials exceed the array is refused."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import plt_oracle as O
from paper_2510_24824_amd import binding as B, synth

pytestmark = pytest.mark.gpu


def _case(Bn, L, Hq, Hkv, D, N, w, seed, dtype=B.PLT_BF16):
    a = synth.make_attn_inputs(Bn, L, Hq, Hkv, D, N, w, seed, bf16=True)
    return a, B.AttnDecode(dtype, a["q"], a["k_share"], a["v_share"], a["k_ring"], a["v_ring"], a["z"])


def test_static_scratch_entry_matches_workspace_entry_twice_second_smaller():
    big = _case(4, 3, 16, 4, 128, 700, 64, 31)        # 16 streams: the stream is split over workgroups (partials used)
    small = _case(2, 2, 8, 2, 64, 90, 16, 32)         # fewer, shorter streams, other head size: reuses the same array
    for (a, ad), n_splits in ((big, 0), (small, 0), (big, 3), (small, 2)):
        y_ref = ad.run(n_splits=n_splits).clone()
        y_st = ad.run_static(n_splits=n_splits).clone()
        torch.cuda.synchronize()
        assert torch.equal(y_ref.view(torch.int16), y_st.view(torch.int16))       # same kernels, same split count: same bits
        ref = O.decode_attention(a["q"], a["k_share"], a["v_share"], a["k_ring"], a["v_ring"], a["z"])
        err = float(np.max(np.abs(y_st.float().cpu().numpy() - ref)))
        assert err <= 2e-2, err


def test_static_scratch_entry_float_and_limits():
    a = synth.make_attn_inputs(2, 2, 4, 2, 64, 40, 8, 33, bf16=False)
    ad = B.AttnDecode(B.PLT_F32, a["q"], a["k_share"], a["v_share"], a["k_ring"], a["v_ring"], a["z"])
    y_ref = ad.run().clone(); y_st = ad.run_static().clone()
    torch.cuda.synchronize()
    assert torch.equal(y_ref, y_st)
    ref = O.decode_attention(a["q"], a["k_share"], a["v_share"], a["k_ring"], a["v_ring"], a["z"])
    assert float(np.max(np.abs(y_st.cpu().numpy() - ref))) <= 1e-5
    # partials beyond the array: refused with a clear error, nothing launched (the pointers are never touched)
    lib = B.lib()
    one = torch.zeros(256, dtype=torch.uint8, device="cuda")
    p = C.c_void_p(one.data_ptr())
    rc = lib.plt_attn_decode_static(B.PLT_BF16, 64, 2, 16, 16, 128, 2048, 2048, 64, 64, p, p, p, p, p, p, p, 4,
                                    C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == -2 and b"scratch" in lib.plt_last_error()
