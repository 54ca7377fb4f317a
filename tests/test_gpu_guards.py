"""Guard rails around the HIP path, through the C ABI:

* canaries -- every output buffer (and the workspace) of every entry point sits between two
  poisoned pads that must come back untouched: an out-of-bounds store that lands in a neighbouring
  allocation would otherwise go unseen;
* a seeded sweep of random shapes through the matrix-core attention kernels against the oracle,
  stopping at the first mismatch: the tripwire for their hand-scheduled instruction groups
  (results of matrix-core instructions issued from inline assembly are invisible to the
  compiler's hazard tracking, so a broken spacing would show up as wrong numbers here);
* the same kind of sweep through the decode entry points, with the length mixes that stress the
  even split of the packed own caches;
* the forward pass run twice gives the same bits, and the matrix-core kernels agree with the
  fp32 vector kernels on a problem with a real softmax.
"""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import cartridge_oracle as orc
from paper_2506_06266_amd import binding as cb
from paper_2506_06266_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
PAD = 1024          # bytes of poison on either side (a multiple of 256: interior stays aligned)
POISON = 0xA5


def to_np(t):
    return t.detach().to("cpu", torch.float64).numpy()


def rel_err(x, ref):
    x, ref = np.asarray(x, np.float64), np.asarray(ref, np.float64)
    assert x.shape == ref.shape and np.isfinite(x).all()
    return float(np.abs(x - ref).max() / max(np.abs(ref).max(), 1e-300))


class Guarded:
    """Tensors carved out of poisoned byte buffers; check() asserts every pad is intact."""

    def __init__(self):
        self.bufs = []

    def empty(self, shape, dtype):
        n = int(np.prod(shape)) * torch.empty(0, dtype=dtype).element_size()
        n_al = (n + 255) // 256 * 256
        raw = torch.full((PAD + n_al + PAD,), POISON, dtype=torch.uint8, device=DEV)
        self.bufs.append((raw, n))
        return raw[PAD:PAD + n].view(dtype).view(*shape)

    def check(self, what):
        for i, (raw, n) in enumerate(self.bufs):
            head, tail = raw[:PAD], raw[PAD + n:]
            assert bool((head == POISON).all()), "%s: buffer %d: bytes BEFORE the output were overwritten" % (what, i)
            assert bool((tail == POISON).all()), "%s: buffer %d: bytes AFTER the output were overwritten" % (what, i)


def _attn_inputs(B, S, Hq, Hkv, P, seed):
    g = torch.Generator().manual_seed(seed)
    rn = lambda *sz, std=1.0: (std * torch.randn(*sz, generator=g)).to(torch.bfloat16)
    return {"q": rn(B, S, Hq, 128, std=0.5), "k": rn(B, S, Hkv, 128, std=0.5), "v": rn(B, S, Hkv, 128),
            "zk": rn(Hkv, P, 128, std=0.5), "zv": rn(Hkv, P, 128), "do": rn(B, S, Hq, 128)}


def test_canaries_attention_fwd_bwd():
    lib = cb.load()
    for impl, (B, S, Hq, Hkv, P) in ((cb.IMPL_MFMA, (2, 331, 4, 2, 77)), (cb.IMPL_MFMA, (1, 65, 2, 1, 0)),
                                     (cb.IMPL_VECTOR, (2, 45, 4, 2, 9))):
        print("case", impl, (B, S, Hq, Hkv, P), flush=True)
        t = {k: v.to(DEV) for k, v in _attn_inputs(B, S, Hq, Hkv, P, 3 * S + P).items()}
        z = (t["zk"], t["zv"]) if P else (None, None)
        gd = Guarded()
        o, lse = gd.empty((B, S, Hq, 128), torch.bfloat16), gd.empty((B, Hq, S), torch.float32)
        d = cb.attn_desc(t["q"], t["k"], P, impl=impl)
        ws = gd.empty((max(lib.cart_attn_bwd_workspace(C.byref(d)), lib.cart_attn_fwd_workspace(C.byref(d)), 16),),
                      torch.uint8)
        cb.cart_attn_fwd(t["q"], t["k"], t["v"], *z, impl=impl, o=o, lse=lse, workspace=ws)
        dq, dk, dv = (gd.empty(x.shape, torch.bfloat16) for x in (t["q"], t["k"], t["v"]))
        dzk = gd.empty((Hkv, P, 128), torch.float32) if P else None
        dzv = gd.empty((Hkv, P, 128), torch.float32) if P else None
        cb.cart_attn_bwd(t["q"], t["k"], t["v"], *z, o, lse, t["do"], impl=impl, d_q=dq, d_k_own=dk, d_v_own=dv,
                         d_z_k=dzk, d_z_v=dzv, workspace=ws)
        torch.cuda.synchronize()
        gd.check("attention impl %d %s" % (impl, (B, S, Hq, Hkv, P)))
        assert torch.isfinite(o.float()).all() and torch.isfinite(dq.float()).all()


def test_canaries_attention_varlen():
    lib = cb.load()
    lens = [100, 1, 300, 37, 201]
    T, Hq, Hkv, P = sum(lens), 4, 2, 70
    t = {k: v.to(DEV) for k, v in _attn_inputs(1, T, Hq, Hkv, P, 9).items()}
    q, k, v, do = (t[n][0] for n in ("q", "k", "v", "do"))
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=DEV)
    gd = Guarded()
    o, lse = gd.empty((T, Hq, 128), torch.bfloat16), gd.empty((Hq, T), torch.float32)
    d = cb.AttnVarlenDesc(T, len(lens), max(lens), Hq, Hkv, 128, P, cb.CART_BF16, 0.0, 0, 0)
    ws = gd.empty((max(lib.cart_attn_varlen_bwd_workspace(C.byref(d)), lib.cart_attn_varlen_fwd_workspace(C.byref(d))),),
                  torch.uint8)
    cb.cart_attn_varlen_fwd(q, k, v, t["zk"], t["zv"], cu, max(lens), o=o, lse=lse, workspace=ws)
    dq, dk, dv = gd.empty(q.shape, torch.bfloat16), gd.empty(k.shape, torch.bfloat16), gd.empty(v.shape, torch.bfloat16)
    dzk, dzv = gd.empty((Hkv, P, 128), torch.float32), gd.empty((Hkv, P, 128), torch.float32)
    cb.cart_attn_varlen_bwd(q, k, v, t["zk"], t["zv"], cu, max(lens), o, lse, do, d_q=dq, d_k_own=dk, d_v_own=dv,
                            d_z_k=dzk, d_z_v=dzv, workspace=ws)
    torch.cuda.synchronize()
    gd.check("packed attention")
    assert torch.isfinite(dq.float()).all() and torch.isfinite(dzk).all()


def test_canaries_loss_and_topk():
    lib = cb.load()
    rng = np.random.default_rng(4)
    for dtype, N, V, K in ((torch.bfloat16, 37, 128256, 20), (torch.bfloat16, 50, 1001, 7), (torch.float32, 33, 777, 5)):
        print("case", dtype, N, V, K, flush=True)
        z = torch.tensor(rng.normal(0, 3, (N, V)), dtype=dtype, device=DEV)
        idx = torch.tensor(np.stack([rng.choice(V, K, replace=False) for _ in range(N)]).astype(np.int32), device=DEV)
        w = rng.normal(0, 1, (N, K))
        lp = torch.tensor((w - np.log(np.exp(w).sum(1, keepdims=True)) + np.log(0.9)).astype(np.float32), device=DEV)
        for mode in (cb.KL_TOPK, cb.KL_REST):
            gd = Guarded()
            dl, loss, row = gd.empty((N, V), dtype), gd.empty((1,), torch.float32), gd.empty((N,), torch.float32)
            kd = cb.KlDesc(N, V, K, cb.CART_BF16 if dtype == torch.bfloat16 else cb.CART_F32, 0.1, mode)
            ws = gd.empty((lib.cart_kl_workspace(C.byref(kd)),), torch.uint8)
            cb.cart_distill_kl_fwd_bwd(z, idx, lp, 0.1, mode=mode, d_logits=dl, loss=loss, row_kl=row, workspace=ws)
            cb.cart_distill_kl_fwd_bwd(z, idx, lp, 0.1, mode=mode, d_logits=dl, loss=loss, workspace=ws)
            torch.cuda.synchronize()
            gd.check("loss %s N%d V%d mode %d" % (dtype, N, V, mode))
            assert torch.isfinite(loss).all()
        gd = Guarded()
        ti, tl = gd.empty((N, K), torch.int32), gd.empty((N, K), torch.float32)
        cb.cart_teacher_topk(z, K, teacher_idx=ti, teacher_logp=tl)
        torch.cuda.synchronize()
        gd.check("top-k %s N%d V%d" % (dtype, N, V))
        assert int(ti.min()) >= 0 and int(ti.max()) < V


def test_canaries_decode_entry_points():
    lib = cb.load()
    g = torch.Generator().manual_seed(8)
    rn = lambda *sz, std=1.0: (std * torch.randn(*sz, generator=g)).to(torch.bfloat16).to(DEV)
    for B, Hq, Hkv, P, max_len in ((37, 8, 2, 700, 333), (3, 32, 8, 33, 5000), (2, 4, 4, 0, 70)):
        print("case", (B, Hq, Hkv, P, max_len), flush=True)
        lens = torch.randint(1, max_len + 1, (B,), generator=g)
        lens[0] = max_len
        cu = torch.zeros(B + 1, dtype=torch.int32)
        cu[1:] = torch.cumsum(lens, 0)
        T = int(cu[-1])
        cu = cu.to(DEV)
        q, k, v = rn(B, Hq, 128, std=0.3), rn(T, Hkv, 128, std=0.3), rn(T, Hkv, 128)
        zk, zv = (rn(Hkv, P, 128, std=0.3), rn(Hkv, P, 128)) if P else (None, None)
        gd = Guarded()
        o, lse = gd.empty((B, Hq, 128), torch.bfloat16), gd.empty((B, Hq), torch.float32)
        dd = cb.DecodeDesc(B, Hq, Hkv, 128, P, T, max_len, cb.CART_BF16, 0.0, cb.IMPL_AUTO)
        ws = gd.empty((max(lib.cart_decode_workspace(C.byref(dd)), 16),), torch.uint8)
        cb.cart_decode(q, zk, zv, k, v, cu, max_len, o=o, lse=lse, workspace=ws)
        o2, lse2 = gd.empty((B, Hq, 128), torch.bfloat16), gd.empty((B, Hq), torch.float32)
        cb.cart_decode_static(q, zk, zv, k, v, cu, max_len, o=o2, lse=lse2)
        # composed: the same prefix in two segments plus a private cartridge for every other request
        if P:
            cut = P // 3
            shared = [(zk[:, :cut].contiguous(), zv[:, :cut].contiguous()), (zk[:, cut:].contiguous(), zv[:, cut:].contiguous())]
            pool_k, pool_v = rn(2, Hkv, 130, 128, std=0.3), rn(2, Hkv, 130, 128)
            cart_id = (torch.arange(B) % 3 - 1).to(torch.int32).to(DEV)
            o3, lse3 = gd.empty((B, Hq, 128), torch.bfloat16), gd.empty((B, Hq), torch.float32)
            segs = (cb.Segment * 2)(*[cb.Segment(a.data_ptr(), b.data_ptr(), a.shape[1]) for a, b in shared])
            cd = cb.DecodeComposedDesc(B, Hq, Hkv, 128, 2, 2, 130, T, max_len, cb.CART_BF16, 0.0)
            ws3 = gd.empty((lib.cart_decode_composed_workspace(C.byref(cd), segs),), torch.uint8)
            cb.cart_decode_composed(q, shared, pool_k, pool_v, cart_id, k, v, cu, max_len, o=o3, lse=lse3, workspace=ws3)
        torch.cuda.synchronize()
        gd.check("decode %s" % ((B, Hq, Hkv, P, max_len),))
        assert torch.equal(o, o2) and torch.isfinite(o.float()).all()


def test_random_shape_sweep_of_the_matrix_core_attention_kernels():
    """About fifty seeded random shapes (S <= 700, P <= 300, every head grouping the kernels take);
    forward and backward against the oracle on every element, stopping at the first mismatch."""
    rng = np.random.default_rng(20250606)
    n_cases = 48
    for case in range(n_cases):
        B = int(rng.integers(1, 4))
        Hkv = int(rng.choice([1, 2, 3]))
        G = int(rng.choice([1, 2, 4, 8]))
        S = int(rng.choice([rng.integers(1, 66), rng.integers(60, 330), rng.integers(300, 701)]))
        P = int(rng.choice([0, rng.integers(1, 70), rng.integers(60, 301)]))
        if B * S * Hkv * G > 6000:          # keep the oracle's share of the test to seconds
            B, G = 1, min(G, 2)
        sharp = bool(rng.integers(0, 2))    # scores of order one (a real softmax) or of order 0.1
        t = _attn_inputs(B, S, Hkv * G, Hkv, P, 1000 + case)
        if sharp:
            t["q"], t["k"], t["zk"] = (x * 2.5 for x in (t["q"], t["k"], t["zk"]))
        n = {k: to_np(v) for k, v in t.items()}
        o_ref, lse_ref = orc.attn_fwd(n["q"], n["k"], n["v"], n["zk"], n["zv"])
        g_ref = orc.attn_bwd(n["q"], n["k"], n["v"], n["zk"], n["zv"], n["do"])
        d = {k: v.to(DEV) for k, v in t.items()}
        z = (d["zk"], d["zv"]) if P else (None, None)
        o, lse = cb.cart_attn_fwd(d["q"], d["k"], d["v"], *z, impl=cb.IMPL_MFMA)
        grads = cb.cart_attn_bwd(d["q"], d["k"], d["v"], *z, o, lse, d["do"], impl=cb.IMPL_MFMA)
        torch.cuda.synchronize()
        errs = {"o": rel_err(to_np(o), o_ref), "lse": rel_err(to_np(lse), lse_ref)}
        for nm, x, r in list(zip(["d_q", "d_k_own", "d_v_own", "d_z_k", "d_z_v"], grads, g_ref))[: 3 if P == 0 else 5]:
            if np.abs(r).max() < 1e-12:
                assert np.abs(to_np(x)).max() < 1e-2
                continue
            errs[nm] = rel_err(to_np(x), r)
        worst = max(errs.values())
        print("sweep %2d  B%d S%d Hq%d Hkv%d P%d sharp=%d  worst %.2e" % (case, B, S, Hkv * G, Hkv, P, sharp, worst), flush=True)
        assert worst <= 2e-2, (case, (B, S, Hkv * G, Hkv, P), errs)


def test_random_shape_sweep_of_the_decode_kernels():
    """Forty seeded random decode problems against the oracle, every element: request counts from 1
    to 300, every head grouping, prefixes from none to ragged, and the length mixes that stress the
    split of the packed own caches -- all requests one token long, one request as long as all
    others together, lengths around the 32-row step and around a range boundary; the composed
    entry point on every third case (two shared segments, a private cartridge for some requests)
    and the static-scratch entry point on every case (bit-equal with the workspace one)."""
    lib = cb.load()
    rng = np.random.default_rng(20250607)
    g = torch.Generator().manual_seed(77)
    rn = lambda *sz, std=1.0: (std * torch.randn(*sz, generator=g)).to(torch.bfloat16)
    for case in range(40):
        Hkv = int(rng.choice([1, 2, 3, 8]))
        G = int(rng.choice([1, 2, 4, 7]))
        B = int(rng.choice([1, 2, rng.integers(3, 40), rng.integers(40, 301)]))
        P = int(rng.choice([0, rng.integers(1, 40), rng.integers(33, 200), 257]))
        mix = int(rng.integers(0, 5))
        if mix == 0:   lens = np.ones(B, dtype=np.int64)
        elif mix == 1: lens = rng.integers(1, 70, B)
        elif mix == 2: lens = np.where(rng.random(B) < 0.15, rng.integers(200, 900, B), rng.integers(1, 5, B))
        elif mix == 3: lens = rng.choice([31, 32, 33, 63, 64, 65, 1], B)
        else:
            lens = rng.integers(1, 20, B)
            lens[int(rng.integers(0, B))] = int(lens.sum()) + 300        # one request as long as all the others
        if int(lens.sum()) * Hkv > 60000:                               # keep the oracle's share to seconds
            lens = np.minimum(lens, 64)
        max_len = int(lens.max())
        cu_np = np.zeros(B + 1, dtype=np.int64)
        cu_np[1:] = np.cumsum(lens)
        T = int(cu_np[-1])
        q, k, v = rn(B, Hkv * G, 128, std=0.6), rn(T, Hkv, 128, std=0.6), rn(T, Hkv, 128)
        zk, zv = (rn(Hkv, P, 128, std=0.6), rn(Hkv, P, 128)) if P else (None, None)
        cu = torch.from_numpy(cu_np).to(torch.int32).to(DEV)
        dz = (zk.to(DEV), zv.to(DEV)) if P else (None, None)
        print("decode sweep %2d  B%d Hq%d Hkv%d P%d T%d max_len%d mix%d" % (case, B, Hkv * G, Hkv, P, T, max_len, mix), flush=True)
        o, lse = cb.cart_decode(q.to(DEV), *dz, k.to(DEV), v.to(DEV), cu, max_len)
        dd = cb.DecodeDesc(B, Hkv * G, Hkv, 128, P, T, max_len, cb.CART_BF16, 0.0, cb.IMPL_AUTO)
        fits = lib.cart_decode_workspace(C.byref(dd)) <= lib.cart_decode_static_capacity()
        o2, lse2 = cb.cart_decode_static(q.to(DEV), *dz, k.to(DEV), v.to(DEV), cu, max_len) if fits else (o, lse)
        torch.cuda.synchronize()
        zk_n = to_np(zk) if P else np.zeros((Hkv, 0, 128))
        zv_n = to_np(zv) if P else np.zeros((Hkv, 0, 128))
        o_ref, lse_ref = orc.decode(to_np(q), zk_n, zv_n, to_np(k), to_np(v), cu_np)
        errs = {"o": rel_err(to_np(o), o_ref), "lse": rel_err(to_np(lse), lse_ref)}
        assert max(errs.values()) <= 2e-2, (case, errs)
        assert torch.equal(o, o2) and torch.equal(lse, lse2), case
        if case % 3 == 0 and P >= 2:
            cut = max(1, P // 3)
            shared = [(zk[:, :cut].contiguous().to(DEV), zv[:, :cut].contiguous().to(DEV)),
                      (zk[:, cut:].contiguous().to(DEV), zv[:, cut:].contiguous().to(DEV))]
            pool_p = int(rng.choice([1, 40, 300]))
            pool_k, pool_v = rn(2, Hkv, pool_p, 128, std=0.6), rn(2, Hkv, pool_p, 128)
            cart_id = (torch.arange(B) % 3 - 1).to(torch.int32)
            o3, lse3 = cb.cart_decode_composed(q.to(DEV), shared, pool_k.to(DEV), pool_v.to(DEV), cart_id.to(DEV),
                                               k.to(DEV), v.to(DEV), cu, max_len)
            torch.cuda.synchronize()
            o3_ref, lse3_ref = orc.decode_composed(to_np(q), [(to_np(a), to_np(b)) for a, b in shared], to_np(pool_k),
                                                   to_np(pool_v), cart_id.numpy(), to_np(k), to_np(v), cu_np)
            errs = {"o": rel_err(to_np(o3), o3_ref), "lse": rel_err(to_np(lse3), lse3_ref)}
            assert max(errs.values()) <= 2e-2, (case, "composed", errs)


def test_forward_twice_same_bits_and_matrix_core_vs_vector_kernels():
    cfg = synth.ATTN_CONFIGS["sharp"]
    g = {k: v.to(DEV) for k, v in synth.attn_inputs(cfg).items()}
    args = (g["q"], g["k_own"], g["v_own"], g["z_k"], g["z_v"])
    o1, l1 = cb.cart_attn_fwd(*args, impl=cb.IMPL_MFMA)
    o2, l2 = cb.cart_attn_fwd(*args, impl=cb.IMPL_MFMA)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
    ov, lv = cb.cart_attn_fwd(*args, impl=cb.IMPL_VECTOR)
    gm = cb.cart_attn_bwd(*args, o1, l1, g["d_o"], impl=cb.IMPL_MFMA)
    gv = cb.cart_attn_bwd(*args, ov, lv, g["d_o"], impl=cb.IMPL_VECTOR)
    torch.cuda.synchronize()
    e = {"o": rel_err(to_np(o1), to_np(ov)), "lse": rel_err(to_np(l1), to_np(lv))}
    for nm, a, b in zip(["d_q", "d_k_own", "d_v_own", "d_z_k", "d_z_v"], gm, gv):
        e[nm] = rel_err(to_np(a), to_np(b))
    print("matrix-core vs vector kernels", e, flush=True)
    for k, x in e.items():
        assert x <= 2e-2, (k, x)
