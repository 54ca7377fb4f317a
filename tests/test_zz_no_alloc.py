"""cart_decode_static (the decode step for callers that cannot allocate: its partial results
live in the library's own per-GPU device array) against cart_decode on the same inputs, through
the C ABI: two calls in a row, the second on a smaller problem, each also checked against the
fp64 oracle; then the size limit and the error paths."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import cartridge_oracle as orc
from paper_2506_06266_amd import binding as cb
from paper_2506_06266_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def to_np(t):
    return t.detach().to("cpu", torch.float64).numpy()


def rel_err(x, r):
    return float(np.abs(x - r).max() / np.abs(r).max())


def _case(seed, B, Hq, Hkv, P, max_len):
    g = torch.Generator().manual_seed(seed)
    D = 128
    rn = lambda *sz, std=1.0: (std * torch.randn(*sz, generator=g)).to(torch.bfloat16)
    lens = torch.randint(1, max_len + 1, (B,), generator=g)
    lens[0] = max_len
    cu = torch.zeros(B + 1, dtype=torch.int32)
    cu[1:] = torch.cumsum(lens, 0)
    T = int(cu[-1])
    return {"q": rn(B, Hq, D, std=0.3), "z_k": rn(Hkv, P, D, std=0.3), "z_v": rn(Hkv, P, D),
            "k_own": rn(T, Hkv, D, std=0.3), "v_own": rn(T, Hkv, D), "cu": cu, "max_len": max_len}


def _both(c):
    g = {k: (v.to(DEV) if torch.is_tensor(v) else v) for k, v in c.items()}
    # poison the outputs so that a call that writes nothing cannot pass
    o_s = torch.full_like(g["q"], float("nan"))
    lse_s = torch.full((g["q"].shape[0], g["q"].shape[1]), float("nan"), dtype=torch.float32, device=DEV)
    cb.cart_decode_static(g["q"], g["z_k"], g["z_v"], g["k_own"], g["v_own"], g["cu"], c["max_len"], o=o_s, lse=lse_s)
    torch.cuda.synchronize()
    o_w, lse_w = cb.cart_decode(g["q"], g["z_k"], g["z_v"], g["k_own"], g["v_own"], g["cu"], c["max_len"])
    torch.cuda.synchronize()
    o_ref, lse_ref = orc.decode(to_np(c["q"]), to_np(c["z_k"]), to_np(c["z_v"]), to_np(c["k_own"]),
                                to_np(c["v_own"]), c["cu"].numpy())
    return o_s, lse_s, o_w, lse_w, o_ref, lse_ref


def test_static_scratch_decode_matches_workspace_decode_twice_in_a_row():
    cb.load()
    # the second call is smaller in every dimension that sizes the scratch use
    for c in (_case(11, 24, 32, 8, 1500, 700), _case(12, 5, 8, 2, 200, 90)):
        print("case B=%d P=%d" % (c["q"].shape[0], c["z_k"].shape[1]), flush=True)
        o_s, lse_s, o_w, lse_w, o_ref, lse_ref = _both(c)
        # same kernels, same plan, same arithmetic: bit-identical to the workspace entry point
        assert torch.equal(o_s, o_w)
        assert torch.equal(lse_s, lse_w)
        # and within the bf16 bar of the oracle
        assert rel_err(to_np(o_s), o_ref) <= 2e-2
        assert rel_err(to_np(lse_s), lse_ref) <= 2e-2


def test_static_scratch_decode_refuses_what_does_not_fit():
    lib = cb.load()
    cap = lib.cart_decode_static_capacity()
    assert cap == 32 << 20
    # 4096 requests x 32 heads: the partial results alone exceed the array
    d = cb.DecodeDesc(4096, 32, 8, 128, 8192, 4096 * 16, 1024, cb.CART_BF16, 0.0, cb.IMPL_AUTO)
    assert lib.cart_decode_workspace(C.byref(d)) > cap
    p = 0x1000
    assert lib.cart_decode_static(C.byref(d), p, p, p, p, p, p, p, p, None) == 4      # CART_ERR_WORKSPACE
    # fp32 is served by the vector kernels, which this entry point does not offer
    d32 = cb.DecodeDesc(4, 8, 2, 64, 16, 64, 32, cb.CART_F32, 0.0, cb.IMPL_AUTO)
    assert lib.cart_decode_static(C.byref(d32), p, p, p, p, p, p, p, p, None) == 3    # CART_ERR_UNSUPPORTED
    ok = cb.DecodeDesc(4, 8, 2, 128, 16, 64, 32, cb.CART_BF16, 0.0, cb.IMPL_AUTO)
    assert lib.cart_decode_static(C.byref(ok), None, p, p, p, p, p, p, p, None) == 1  # CART_ERR_NULL
