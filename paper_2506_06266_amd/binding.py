"""ctypes binding over libcartridge.so (the C ABI declared in include/cartridge.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
PyTorch supplies device memory and the stream.  There is no fallback: if the library is
missing, or a call returns a non-zero status, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcartridge.so")

CART_F32, CART_BF16 = 0, 1
IMPL_AUTO, IMPL_VECTOR, IMPL_MFMA = 0, 1, 2
STATUS_NAMES = ["CART_OK", "CART_ERR_NULL", "CART_ERR_SHAPE", "CART_ERR_UNSUPPORTED",
                "CART_ERR_WORKSPACE", "CART_ERR_LAUNCH", "CART_ERR_ALIGN"]

EXPORTS = ["cart_attn_fwd_workspace", "cart_attn_bwd_workspace", "cart_kl_workspace",
           "cart_decode_workspace", "cart_attn_fwd", "cart_attn_bwd", "cart_distill_kl_fwd_bwd",
           "cart_decode", "cart_decode_composed_workspace", "cart_decode_composed", "cart_teacher_topk",
           "cart_attn_varlen_fwd_workspace", "cart_attn_varlen_bwd_workspace", "cart_attn_varlen_fwd",
           "cart_attn_varlen_bwd", "cart_trace_events", "cart_calib_mfma", "cart_calib_copy",
           "cart_calib_read", "cart_decode_static", "cart_decode_static_capacity",
           "cart_status_str", "cart_version"]


class AttnDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("S", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32),
                ("D", C.c_int32), ("P", C.c_int32), ("dtype", C.c_int), ("softmax_scale", C.c_float),
                ("n_frozen", C.c_int32), ("dz_accumulate", C.c_int32), ("impl", C.c_int)]


class AttnVarlenDesc(C.Structure):
    _fields_ = [("T", C.c_int32), ("B", C.c_int32), ("max_seqlen", C.c_int32), ("Hq", C.c_int32),
                ("Hkv", C.c_int32), ("D", C.c_int32), ("P", C.c_int32), ("dtype", C.c_int),
                ("softmax_scale", C.c_float), ("n_frozen", C.c_int32), ("dz_accumulate", C.c_int32)]


class KlDesc(C.Structure):
    _fields_ = [("N", C.c_int32), ("V", C.c_int32), ("K", C.c_int32), ("logits_dtype", C.c_int),
                ("scale", C.c_float), ("mode", C.c_int)]


class TopkDesc(C.Structure):
    _fields_ = [("N", C.c_int32), ("V", C.c_int32), ("K", C.c_int32), ("logits_dtype", C.c_int)]


class Segment(C.Structure):
    _fields_ = [("z_k", C.c_void_p), ("z_v", C.c_void_p), ("p", C.c_int32)]


class DecodeComposedDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
                ("n_shared", C.c_int32), ("n_pool", C.c_int32), ("pool_p", C.c_int32),
                ("total_own_tokens", C.c_int32), ("max_own_len", C.c_int32), ("dtype", C.c_int),
                ("softmax_scale", C.c_float)]


class DecodeDesc(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
                ("P", C.c_int32), ("total_own_tokens", C.c_int32), ("max_own_len", C.c_int32),
                ("dtype", C.c_int), ("softmax_scale", C.c_float), ("impl", C.c_int)]


class CartridgeError(RuntimeError):
    def __init__(self, status: int, what: str):
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__("%s failed: %s (%s)" % (what, name, status_str(status)))
        self.status = status


_lib = None


def load() -> C.CDLL:
    """Loads the in-tree library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s not found: build it with `python -m paper_2506_06266_amd.build`" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, sz = C.c_void_p, C.c_size_t
    for name, desc in (("cart_attn_fwd_workspace", AttnDesc), ("cart_attn_bwd_workspace", AttnDesc),
                       ("cart_kl_workspace", KlDesc), ("cart_decode_workspace", DecodeDesc),
                       ("cart_attn_varlen_fwd_workspace", AttnVarlenDesc),
                       ("cart_attn_varlen_bwd_workspace", AttnVarlenDesc)):
        f = getattr(lib, name)
        f.restype, f.argtypes = sz, [C.POINTER(desc)]
    lib.cart_attn_fwd.restype = C.c_int
    lib.cart_attn_fwd.argtypes = [C.POINTER(AttnDesc)] + [vp] * 8 + [sz, vp]
    lib.cart_attn_bwd.restype = C.c_int
    lib.cart_attn_bwd.argtypes = [C.POINTER(AttnDesc)] + [vp] * 14 + [sz, vp]
    lib.cart_attn_varlen_fwd.restype = C.c_int
    lib.cart_attn_varlen_fwd.argtypes = [C.POINTER(AttnVarlenDesc)] + [vp] * 9 + [sz, vp]
    lib.cart_attn_varlen_bwd.restype = C.c_int
    lib.cart_attn_varlen_bwd.argtypes = [C.POINTER(AttnVarlenDesc)] + [vp] * 15 + [sz, vp]
    lib.cart_distill_kl_fwd_bwd.restype = C.c_int
    lib.cart_distill_kl_fwd_bwd.argtypes = [C.POINTER(KlDesc)] + [vp] * 7 + [sz, vp]
    lib.cart_decode.restype = C.c_int
    lib.cart_decode.argtypes = [C.POINTER(DecodeDesc)] + [vp] * 9 + [sz, vp]
    lib.cart_decode_static.restype = C.c_int
    lib.cart_decode_static.argtypes = [C.POINTER(DecodeDesc)] + [vp] * 9
    lib.cart_decode_static_capacity.restype, lib.cart_decode_static_capacity.argtypes = sz, []
    lib.cart_teacher_topk.restype = C.c_int
    lib.cart_teacher_topk.argtypes = [C.POINTER(TopkDesc), vp, vp, vp, vp]
    lib.cart_decode_composed_workspace.restype = sz
    lib.cart_decode_composed_workspace.argtypes = [C.POINTER(DecodeComposedDesc), C.POINTER(Segment)]
    lib.cart_decode_composed.restype = C.c_int
    lib.cart_decode_composed.argtypes = [C.POINTER(DecodeComposedDesc), vp, C.POINTER(Segment)] + [vp] * 9 + [sz, vp]
    lib.cart_trace_events.restype = C.c_int
    lib.cart_trace_events.argtypes = [C.POINTER(C.c_void_p), C.c_int32]
    lib.cart_calib_mfma.restype = C.c_double
    lib.cart_calib_mfma.argtypes = [vp, C.c_int32, C.c_int32, vp]
    lib.cart_calib_copy.restype = C.c_int
    lib.cart_calib_copy.argtypes = [vp, vp, sz, vp]
    lib.cart_calib_read.restype = C.c_int
    lib.cart_calib_read.argtypes = [vp, sz, vp, vp]
    lib.cart_status_str.restype, lib.cart_status_str.argtypes = C.c_char_p, [C.c_int]
    lib.cart_version.restype, lib.cart_version.argtypes = C.c_int, []
    _lib = lib
    return lib


def status_str(status: int) -> str:
    return load().cart_status_str(status).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return CART_F32
    if t.dtype == torch.bfloat16:
        return CART_BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors handed to libcartridge must be contiguous device tensors")
    return t.data_ptr() if t.numel() > 0 else None


def _stream(stream) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def _workspace(nbytes: int, workspace: Optional[torch.Tensor], device) -> Optional[torch.Tensor]:
    if workspace is not None:
        return workspace
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def _check(status: int, what: str):
    if status != 0:
        raise CartridgeError(status, what)


# ------------------------------------------------------------------------------------------------
def attn_desc(q: torch.Tensor, k_own: torch.Tensor, p: int, scale: float = 0.0, n_frozen: int = 0,
              dz_accumulate: bool = False, impl: int = IMPL_AUTO) -> AttnDesc:
    B, S, Hq, D = q.shape
    return AttnDesc(B, S, Hq, k_own.shape[2], D, p, _dtype_code(q), scale, n_frozen,
                    int(dz_accumulate), impl)


def cart_attn_fwd(q, k_own, v_own, z_k, z_v, *, scale: float = 0.0, impl: int = IMPL_AUTO,
                  o=None, lse=None, workspace=None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """q [B,S,Hq,D]; k_own, v_own [B,S,Hkv,D]; z_k, z_v [Hkv,P,D] -> (o [B,S,Hq,D], lse [B,Hq,S])."""
    lib = load()
    p = 0 if z_k is None else z_k.shape[1]
    d = attn_desc(q, k_own, p, scale, impl=impl)
    B, S, Hq, D = q.shape
    o = torch.empty_like(q) if o is None else o
    lse = torch.empty(B, Hq, S, dtype=torch.float32, device=q.device) if lse is None else lse
    need = lib.cart_attn_fwd_workspace(C.byref(d))
    ws = _workspace(need, workspace, q.device)
    st = lib.cart_attn_fwd(C.byref(d), _ptr(q), _ptr(k_own), _ptr(v_own), _ptr(z_k), _ptr(z_v),
                           _ptr(o), _ptr(lse), _ptr(ws), 0 if ws is None else ws.numel(),
                           _stream(stream))
    _check(st, "cart_attn_fwd")
    return o, lse


def cart_attn_bwd(q, k_own, v_own, z_k, z_v, o, lse, d_o, *, scale: float = 0.0, n_frozen: int = 0,
                  d_z_k=None, d_z_v=None, dz_accumulate: bool = False, impl: int = IMPL_AUTO,
                  d_q=None, d_k_own=None, d_v_own=None, workspace=None, stream=None):
    """Returns (d_q, d_k_own, d_v_own, d_z_k, d_z_v); d_z_* are fp32 [Hkv,P,D]."""
    lib = load()
    p = 0 if z_k is None else z_k.shape[1]
    d = attn_desc(q, k_own, p, scale, n_frozen, dz_accumulate, impl)
    d_q = torch.empty_like(q) if d_q is None else d_q
    d_k_own = torch.empty_like(k_own) if d_k_own is None else d_k_own
    d_v_own = torch.empty_like(v_own) if d_v_own is None else d_v_own
    if p > 0:
        if d_z_k is None:
            if dz_accumulate:
                raise ValueError("dz_accumulate needs d_z_k / d_z_v")
            d_z_k = torch.empty(z_k.shape, dtype=torch.float32, device=q.device)
            d_z_v = torch.empty(z_v.shape, dtype=torch.float32, device=q.device)
    need = lib.cart_attn_bwd_workspace(C.byref(d))
    ws = _workspace(need, workspace, q.device)
    st = lib.cart_attn_bwd(C.byref(d), _ptr(q), _ptr(k_own), _ptr(v_own), _ptr(z_k), _ptr(z_v),
                           _ptr(o), _ptr(lse), _ptr(d_o), _ptr(d_q), _ptr(d_k_own), _ptr(d_v_own),
                           _ptr(d_z_k), _ptr(d_z_v), _ptr(ws), 0 if ws is None else ws.numel(),
                           _stream(stream))
    _check(st, "cart_attn_bwd")
    return d_q, d_k_own, d_v_own, d_z_k, d_z_v


def cart_attn_varlen_fwd(q, k_own, v_own, z_k, z_v, cu_seqlens, max_seqlen: int, *, scale: float = 0.0,
                         o=None, lse=None, workspace=None, stream=None):
    """Packed batch: q [T,Hq,D]; k_own, v_own [T,Hkv,D]; z_k, z_v [Hkv,P,D]; cu_seqlens [B+1] int32
    (device) -> (o [T,Hq,D], lse [Hq,T])."""
    lib = load()
    T, Hq, D = q.shape
    p = 0 if z_k is None else z_k.shape[1]
    d = AttnVarlenDesc(T, cu_seqlens.numel() - 1, max_seqlen, Hq, k_own.shape[1], D, p, _dtype_code(q), scale, 0, 0)
    o = torch.empty_like(q) if o is None else o
    lse = torch.empty(Hq, T, dtype=torch.float32, device=q.device) if lse is None else lse
    need = lib.cart_attn_varlen_fwd_workspace(C.byref(d))
    ws = _workspace(need, workspace, q.device)
    st = lib.cart_attn_varlen_fwd(C.byref(d), _ptr(q), _ptr(k_own), _ptr(v_own), _ptr(z_k), _ptr(z_v),
                                  _ptr(cu_seqlens), _ptr(o), _ptr(lse), _ptr(ws),
                                  0 if ws is None else ws.numel(), _stream(stream))
    _check(st, "cart_attn_varlen_fwd")
    return o, lse


def cart_attn_varlen_bwd(q, k_own, v_own, z_k, z_v, cu_seqlens, max_seqlen: int, o, lse, d_o, *,
                         scale: float = 0.0, n_frozen: int = 0, d_z_k=None, d_z_v=None,
                         dz_accumulate: bool = False, d_q=None, d_k_own=None, d_v_own=None,
                         workspace=None, stream=None):
    """Returns (d_q, d_k_own, d_v_own [packed], d_z_k, d_z_v [Hkv,P,D] fp32)."""
    lib = load()
    T, Hq, D = q.shape
    p = 0 if z_k is None else z_k.shape[1]
    d = AttnVarlenDesc(T, cu_seqlens.numel() - 1, max_seqlen, Hq, k_own.shape[1], D, p, _dtype_code(q), scale,
                       n_frozen, int(dz_accumulate))
    d_q = torch.empty_like(q) if d_q is None else d_q
    d_k_own = torch.empty_like(k_own) if d_k_own is None else d_k_own
    d_v_own = torch.empty_like(v_own) if d_v_own is None else d_v_own
    if p > 0 and d_z_k is None:
        if dz_accumulate:
            raise ValueError("dz_accumulate needs d_z_k / d_z_v")
        d_z_k = torch.empty(z_k.shape, dtype=torch.float32, device=q.device)
        d_z_v = torch.empty(z_v.shape, dtype=torch.float32, device=q.device)
    need = lib.cart_attn_varlen_bwd_workspace(C.byref(d))
    ws = _workspace(need, workspace, q.device)
    st = lib.cart_attn_varlen_bwd(C.byref(d), _ptr(q), _ptr(k_own), _ptr(v_own), _ptr(z_k), _ptr(z_v),
                                  _ptr(cu_seqlens), _ptr(o), _ptr(lse), _ptr(d_o), _ptr(d_q), _ptr(d_k_own),
                                  _ptr(d_v_own), _ptr(d_z_k), _ptr(d_z_v), _ptr(ws),
                                  0 if ws is None else ws.numel(), _stream(stream))
    _check(st, "cart_attn_varlen_bwd")
    return d_q, d_k_own, d_v_own, d_z_k, d_z_v


KL_TOPK, KL_REST = 0, 1


def cart_distill_kl_fwd_bwd(logits, teacher_idx, teacher_logp, scale: float, *, mode: int = KL_TOPK,
                            d_logits=None, loss=None, row_kl=None, workspace=None, stream=None):
    """logits [N,V]; teacher_idx [N,K] int32; teacher_logp [N,K] fp32 or None (all zero: with
    K = 1 that is next-token cross-entropy on the labels teacher_idx[:,0]) ->
    (loss [1] fp32 device tensor, d_logits [N,V]).  Pass d_logits=logits to work in place."""
    lib = load()
    N, V = logits.shape
    d = KlDesc(N, V, teacher_idx.shape[1], _dtype_code(logits), scale, mode)
    d_logits = torch.empty_like(logits) if d_logits is None else d_logits
    loss = torch.empty(1, dtype=torch.float32, device=logits.device) if loss is None else loss
    need = lib.cart_kl_workspace(C.byref(d))
    ws = _workspace(need, workspace, logits.device)
    st = lib.cart_distill_kl_fwd_bwd(C.byref(d), _ptr(logits), _ptr(teacher_idx), _ptr(teacher_logp),
                                     _ptr(loss), _ptr(d_logits), _ptr(row_kl), _ptr(ws),
                                     0 if ws is None else ws.numel(), _stream(stream))
    _check(st, "cart_distill_kl_fwd_bwd")
    return loss, d_logits


def cart_decode(q, z_k, z_v, k_own, v_own, cu_lens, max_own_len: int, *, scale: float = 0.0,
                impl: int = IMPL_AUTO, o=None, lse=None, workspace=None, stream=None):
    """q [B,Hq,D]; z_k, z_v [Hkv,P,D]; k_own, v_own [T,Hkv,D]; cu_lens [B+1] int32 (device) ->
    (o [B,Hq,D], lse [B,Hq])."""
    lib = load()
    B, Hq, D = q.shape
    p = 0 if z_k is None else z_k.shape[1]
    d = DecodeDesc(B, Hq, k_own.shape[1], D, p, k_own.shape[0], max_own_len, _dtype_code(q), scale, impl)
    o = torch.empty_like(q) if o is None else o
    lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device) if lse is None else lse
    need = lib.cart_decode_workspace(C.byref(d))
    ws = _workspace(need, workspace, q.device)
    st = lib.cart_decode(C.byref(d), _ptr(q), _ptr(z_k), _ptr(z_v), _ptr(k_own), _ptr(v_own),
                         _ptr(cu_lens), _ptr(o), _ptr(lse), _ptr(ws),
                         0 if ws is None else ws.numel(), _stream(stream))
    _check(st, "cart_decode")
    return o, lse


def cart_decode_static(q, z_k, z_v, k_own, v_own, cu_lens, max_own_len: int, *, scale: float = 0.0,
                       o=None, lse=None, stream=None):
    """cart_decode without a workspace: the library's own per-GPU scratch array holds the partial
    results (nothing is allocated by the call itself when o and lse are passed in)."""
    lib = load()
    B, Hq, D = q.shape
    p = 0 if z_k is None else z_k.shape[1]
    d = DecodeDesc(B, Hq, k_own.shape[1], D, p, k_own.shape[0], max_own_len, _dtype_code(q), scale, IMPL_AUTO)
    o = torch.empty_like(q) if o is None else o
    lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device) if lse is None else lse
    st = lib.cart_decode_static(C.byref(d), _ptr(q), _ptr(z_k), _ptr(z_v), _ptr(k_own), _ptr(v_own),
                                _ptr(cu_lens), _ptr(o), _ptr(lse), _stream(stream))
    _check(st, "cart_decode_static")
    return o, lse


def cart_teacher_topk(logits, k: int, *, teacher_idx=None, teacher_logp=None, stream=None):
    """logits [N,V] -> (teacher_idx [N,k] int32, teacher_logp [N,k] fp32), by descending probability."""
    lib = load()
    N, V = logits.shape
    d = TopkDesc(N, V, k, _dtype_code(logits))
    idx = torch.empty(N, k, dtype=torch.int32, device=logits.device) if teacher_idx is None else teacher_idx
    lp = torch.empty(N, k, dtype=torch.float32, device=logits.device) if teacher_logp is None else teacher_logp
    st = lib.cart_teacher_topk(C.byref(d), _ptr(logits), _ptr(idx), _ptr(lp), _stream(stream))
    _check(st, "cart_teacher_topk")
    return idx, lp


def cart_decode_composed(q, shared, pool_k, pool_v, cart_id, k_own, v_own, cu_lens, max_own_len: int, *,
                         scale: float = 0.0, o=None, lse=None, workspace=None, stream=None):
    """q [B,Hq,D]; shared: list of (z_k, z_v) tensors [Hkv,p_s,D] every request attends over;
    pool_k, pool_v [n_pool,Hkv,p_c,D] and cart_id [B] int32 (device; < 0 = none), or None;
    k_own, v_own [T,Hkv,D]; cu_lens [B+1] int32 (device) -> (o [B,Hq,D], lse [B,Hq])."""
    lib = load()
    B, Hq, D = q.shape
    segs = (Segment * max(len(shared), 1))()
    for i, (zk, zv) in enumerate(shared):
        segs[i] = Segment(_ptr(zk), _ptr(zv), zk.shape[1])
    n_pool, pool_p = (0, 0) if pool_k is None else (pool_k.shape[0], pool_k.shape[2])
    d = DecodeComposedDesc(B, Hq, k_own.shape[1], D, len(shared), n_pool, pool_p, k_own.shape[0], max_own_len,
                           _dtype_code(q), scale)
    o = torch.empty_like(q) if o is None else o
    lse = torch.empty(B, Hq, dtype=torch.float32, device=q.device) if lse is None else lse
    need = lib.cart_decode_composed_workspace(C.byref(d), segs)
    ws = _workspace(need, workspace, q.device)
    st = lib.cart_decode_composed(C.byref(d), _ptr(q), segs, _ptr(pool_k), _ptr(pool_v), _ptr(cart_id),
                                  _ptr(k_own), _ptr(v_own), _ptr(cu_lens), _ptr(o), _ptr(lse), _ptr(ws),
                                  0 if ws is None else ws.numel(), _stream(stream))
    _check(st, "cart_decode_composed")
    return o, lse


# ------------------------------------------------------------------------------------------------
def cart_calib_mfma(sink: torch.Tensor, iters: int, wgs_per_cu: int = 1, stream=None) -> float:
    """Enqueues the matrix-core-only loop; returns the flops the launch performs."""
    fl = load().cart_calib_mfma(_ptr(sink), iters, wgs_per_cu, _stream(stream))
    if fl <= 0.0:
        raise CartridgeError(5, "cart_calib_mfma")
    return fl


def cart_calib_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    _check(load().cart_calib_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream(stream)),
           "cart_calib_copy")


def cart_calib_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    _check(load().cart_calib_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream)),
           "cart_calib_read")


class KernelTrace:
    """HIP events recorded by the library at kernel boundaries (cart_trace_events).

    with KernelTrace(6) as tr:  cart_attn_bwd(...);  torch.cuda.synchronize();  tr.intervals_ms()
    """

    def __init__(self, count: int):
        self.count = count
        self._hip = C.CDLL("libamdhip64.so")
        self._hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self._hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self._hip.hipEventDestroy.argtypes = [C.c_void_p]
        self._hip.hipEventQuery.argtypes = [C.c_void_p]
        self.events = (C.c_void_p * count)()
        for i in range(count):
            ev = C.c_void_p()
            if self._hip.hipEventCreate(C.byref(ev)) != 0:
                raise RuntimeError("hipEventCreate failed")
            self.events[i] = ev

    def __enter__(self):
        _check(load().cart_trace_events(self.events, self.count), "cart_trace_events")
        return self

    def __exit__(self, *exc):
        load().cart_trace_events(None, 0)
        return False

    def intervals_ms(self, n: Optional[int] = None):
        """Elapsed ms between consecutive events 0..n (call after synchronising the stream)."""
        n = self.count if n is None else n
        out = []
        for i in range(n - 1):
            ms = C.c_float()
            rc = self._hip.hipEventElapsedTime(C.byref(ms), self.events[i], self.events[i + 1])
            if rc != 0:
                raise RuntimeError("hipEventElapsedTime failed (%d): event %d not recorded?" % (rc, i + 1))
            out.append(ms.value)
        return out

    def close(self):
        for i in range(self.count):
            self._hip.hipEventDestroy(self.events[i])
