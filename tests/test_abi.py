"""The C-ABI library loads, exports every symbol the header declares, and validates its
arguments on the host (no kernel is launched by anything in this file)."""
import ctypes as C
import os
import re

import pytest

from paper_2506_06266_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2506_06266_amd import build
        build.build(force=False)
    return binding.load()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "cartridge.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cart_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings(lib):
    assert lib.cart_version() >= 100
    for code in range(7):
        assert len(binding.status_str(code)) > 0


def test_workspace_queries(lib):
    d = binding.AttnDesc(16, 2048, 32, 8, 128, 4096, binding.CART_BF16, 0.0, 0, 0, binding.IMPL_VECTOR)
    assert lib.cart_attn_fwd_workspace(C.byref(d)) == 0
    assert lib.cart_attn_bwd_workspace(C.byref(d)) >= 16 * 32 * 2048 * 4
    k = binding.KlDesc(16384, 128256, 20, binding.CART_BF16, 1.0 / 16384)
    assert lib.cart_kl_workspace(C.byref(k)) >= 16384 * 4
    bad = binding.AttnDesc(16, 2048, 32, 7, 128, 4096, binding.CART_BF16, 0.0, 0, 0, 0)
    assert lib.cart_attn_bwd_workspace(C.byref(bad)) == 0


def _attn_call(lib, d, ptrs=None, ws=0x1000, ws_bytes=1 << 30):
    ptrs = ptrs or [0x1000] * 7
    return lib.cart_attn_fwd(C.byref(d), *ptrs, ws, ws_bytes, None)


def test_attn_argument_validation_returns_status_without_launching(lib):
    ok = dict(B=2, S=8, Hq=4, Hkv=2, D=64, P=4, dtype=binding.CART_F32, softmax_scale=0.0,
              n_frozen=0, dz_accumulate=0, impl=binding.IMPL_VECTOR)
    def desc(**kw):
        return binding.AttnDesc(**{**ok, **kw})
    assert _attn_call(lib, desc(Hkv=3)) == 2           # Hq % Hkv != 0
    assert _attn_call(lib, desc(B=0)) == 2
    assert _attn_call(lib, desc(P=-1)) == 2
    assert _attn_call(lib, desc(D=512)) == 3
    assert _attn_call(lib, desc(dtype=7)) == 3
    assert _attn_call(lib, desc(impl=binding.IMPL_MFMA)) == 3     # fp32 has no MFMA path
    assert _attn_call(lib, desc(n_frozen=5)) == 2
    assert _attn_call(lib, desc(softmax_scale=-1.0)) == 2
    assert _attn_call(lib, desc(), ptrs=[None] + [0x1000] * 6) == 1
    assert _attn_call(lib, desc(), ptrs=[0x1000] * 3 + [None, 0x1000, 0x1000, 0x1000]) == 1   # z_k with P>0
    assert _attn_call(lib, desc(), ptrs=[0x1004] + [0x1000] * 6) == 6
    assert lib.cart_attn_fwd(None, *([0x1000] * 7), None, 0, None) == 1
    # backward: workspace too small
    d = desc()
    need = lib.cart_attn_bwd_workspace(C.byref(d))
    assert need > 0
    st = lib.cart_attn_bwd(C.byref(d), *([0x1000] * 13), 0x1000, need - 1, None)
    assert st == 4
    st = lib.cart_attn_bwd(C.byref(d), *([0x1000] * 13), None, need, None)
    assert st == 4


def test_kl_and_decode_argument_validation(lib):
    k = binding.KlDesc(4, 10, 20, binding.CART_F32, 1.0)
    assert lib.cart_distill_kl_fwd_bwd(C.byref(k), *([0x1000] * 7), 1 << 20, None) == 2   # K > V
    k = binding.KlDesc(4, 5000, 2000, binding.CART_F32, 1.0)
    assert lib.cart_distill_kl_fwd_bwd(C.byref(k), *([0x1000] * 7), 1 << 20, None) == 3   # K > 1024
    k = binding.KlDesc(4, 100, 5, binding.CART_F32, float("nan"))
    assert lib.cart_distill_kl_fwd_bwd(C.byref(k), *([0x1000] * 7), 1 << 20, None) == 2
    k = binding.KlDesc(4, 100, 5, binding.CART_F32, 1.0, 7)
    assert lib.cart_distill_kl_fwd_bwd(C.byref(k), *([0x1000] * 7), 1 << 20, None) == 3   # unknown mode
    k = binding.KlDesc(4, 100, 5, binding.CART_F32, 1.0)
    args = [0x1000] * 7
    args[3] = None                                       # loss
    assert lib.cart_distill_kl_fwd_bwd(C.byref(k), *args, 1 << 20, None) == 1
    args = [0x1000] * 7
    args[5] = None; args[6] = None                       # no row_kl and no workspace
    assert lib.cart_distill_kl_fwd_bwd(C.byref(k), *args, 0, None) == 4
    d = binding.DecodeDesc(4, 8, 3, 128, 16, 40, 20, binding.CART_BF16, 0.0, 0)
    assert lib.cart_decode(C.byref(d), *([0x1000] * 9), 0, None) == 2     # Hq % Hkv
    d = binding.DecodeDesc(4, 8, 2, 128, 16, 3, 2, binding.CART_BF16, 0.0, 0)
    assert lib.cart_decode(C.byref(d), *([0x1000] * 9), 0, None) == 2     # fewer own rows than requests
    d = binding.DecodeDesc(4, 8, 2, 128, 16, 40, 20, binding.CART_BF16, 0.0, 0)
    args = [0x1000] * 9
    args[5] = None                                       # cu_lens
    assert lib.cart_decode(C.byref(d), *args, 0, None) == 1


def test_varlen_attention_argument_validation(lib):
    mk = lambda **kw: binding.AttnVarlenDesc(**{**dict(T=500, B=3, max_seqlen=300, Hq=8, Hkv=2, D=128, P=64,
                                                       dtype=binding.CART_BF16, softmax_scale=0.0, n_frozen=0,
                                                       dz_accumulate=0), **kw})
    d = mk()
    need_f, need_b = lib.cart_attn_varlen_fwd_workspace(C.byref(d)), lib.cart_attn_varlen_bwd_workspace(C.byref(d))
    # one flag per workgroup of the grid sized for max_seqlen; two row arrays and two partial buffers
    assert need_f >= 2 * 3 * 8 * 4
    assert need_b >= 2 * 500 * 8 * 4 + 2 * 1 * 2 * 64 * 128 * 4
    fwd = lambda d, args, ws=0x1000, n=1 << 30: lib.cart_attn_varlen_fwd(C.byref(d), *args, ws, n, None)
    ok = [0x1000] * 8
    assert fwd(mk(max_seqlen=501), ok) == 2 and fwd(mk(max_seqlen=0), ok) == 2 and fwd(mk(T=0), ok) == 2
    assert fwd(mk(dtype=binding.CART_F32), ok) == 3 and fwd(mk(D=64), ok) == 3
    assert fwd(mk(Hkv=3), ok) == 2
    a = list(ok); a[5] = None                            # cu_seqlens
    assert fwd(d, a) == 1
    assert fwd(d, ok, 0x1000, need_f - 1) == 4
    a = list(ok); a[0] = 0x1004
    assert fwd(d, a) == 6
    assert lib.cart_attn_varlen_bwd(C.byref(d), *([0x1000] * 14), 0x1000, need_b - 1, None) == 4
    a = [0x1000] * 14; a[12] = None                      # d_z_k with P > 0
    assert lib.cart_attn_varlen_bwd(C.byref(d), *a, 0x1000, need_b, None) == 1
    assert lib.cart_attn_varlen_bwd(C.byref(mk(n_frozen=65)), *([0x1000] * 14), 0x1000, need_b, None) == 2
