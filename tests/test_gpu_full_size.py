"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The GPU runs the whole problem.  Attention: the oracle recomputes the forward pass of every KV
group (every element of O and LSE), and the backward pass of two whole KV groups on different
residues of the workgroup-to-XCD rotation (every sequence, their G query heads), which fixes dQ
for those heads, dK_own / dV_own for those KV heads and -- because the sum over the whole batch
is inside the sample -- dZ_k / dZ_v of those heads, every element.  Loss: every row's value and
the scalar against the oracle run in row chunks, the gradient on sampled rows.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from oracle import cartridge_oracle as orc
from paper_2506_06266_amd import binding as cb
from paper_2506_06266_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"
TOL = 2e-2


def rel_err(x, ref) -> float:
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert x.shape == ref.shape and np.isfinite(x).all()
    return float(np.abs(x - ref).max() / np.abs(ref).max())


def elem_err(x, ref, floor=1e-3) -> float:
    """Element-wise relative error with an absolute floor of `floor` x max |ref| in the denominator."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float((np.abs(x - ref) / np.maximum(np.abs(ref), floor * np.abs(ref).max())).max())


def f64(t):
    return t.detach().to("cpu", torch.float64).numpy()


@pytest.mark.parametrize("name,grad_heads", [("cfg2", (5, 0)), ("cfg3", (2, 7))])
def test_attention_full_shape_every_kv_group(name, grad_heads):
    cfg = synth.ATTN_CONFIGS[name]
    print("case", name, "gradients of kv heads", grad_heads, flush=True)
    g = synth.attn_inputs(cfg, DEV)
    o, lse = cb.cart_attn_fwd(g["q"], g["k_own"], g["v_own"], g["z_k"], g["z_v"])
    dq, dk, dv, dzk, dzv = cb.cart_attn_bwd(g["q"], g["k_own"], g["v_own"], g["z_k"], g["z_v"], o, lse, g["d_o"])
    torch.cuda.synchronize()
    G = cfg.Hq // cfg.Hkv
    for hk in range(cfg.Hkv):
        hs = slice(hk * G, (hk + 1) * G)
        q, do = f64(g["q"][:, :, hs]), f64(g["d_o"][:, :, hs])
        k, v = f64(g["k_own"][:, :, hk:hk + 1]), f64(g["v_own"][:, :, hk:hk + 1])
        zk, zv = f64(g["z_k"][hk:hk + 1]), f64(g["z_v"][hk:hk + 1])
        o_ref, lse_ref = orc.attn_fwd(q, k, v, zk, zv)
        pairs = {"o": (f64(o[:, :, hs]), o_ref), "lse": (f64(lse[:, hs]), lse_ref)}
        if hk in grad_heads:
            r = orc.attn_bwd(q, k, v, zk, zv, do)
            pairs.update({"dq": (f64(dq[:, :, hs]), r[0]), "dk": (f64(dk[:, :, hk:hk + 1]), r[1]),
                          "dv": (f64(dv[:, :, hk:hk + 1]), r[2]), "dzk": (f64(dzk[hk:hk + 1]), r[3]),
                          "dzv": (f64(dzv[hk:hk + 1]), r[4])})
        errs = {kk: rel_err(x, rr) for kk, (x, rr) in pairs.items()}
        print(name, "kv head", hk, "max|x-ref|/max|ref|", {kk: "%.2e" % e for kk, e in errs.items()},
              "element-wise (floor 1e-3 max|ref|)", {kk: "%.2e" % elem_err(x, rr) for kk, (x, rr) in pairs.items()},
              flush=True)
        for kk, e in errs.items():
            assert e <= TOL, (name, hk, kk, e)
    # the backward pass is bit-reproducible (no atomics): a second run gives the same bits
    again = cb.cart_attn_bwd(g["q"], g["k_own"], g["v_own"], g["z_k"], g["z_v"], o, lse, g["d_o"])
    torch.cuda.synchronize()
    for a, b in zip((dq, dk, dv, dzk, dzv), again):
        assert torch.equal(a, b)
    # and so is the forward pass
    o2, lse2 = cb.cart_attn_fwd(g["q"], g["k_own"], g["v_own"], g["z_k"], g["z_v"])
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(lse, lse2)


@pytest.mark.parametrize("mode", [cb.KL_TOPK, cb.KL_REST], ids=["topk", "rest"])
def test_distill_kl_full_size_sampled_rows(mode):
    cfg = synth.KL_CONFIGS["cfg4"]
    print("case cfg4 mode", mode, flush=True)
    g = synth.kl_inputs(cfg, DEV)
    row_kl = torch.empty(cfg.N, dtype=torch.float32, device=DEV)
    loss, dl = cb.cart_distill_kl_fwd_bwd(g["logits"], g["teacher_idx"], g["teacher_logp"], cfg.scale, mode=mode,
                                          row_kl=row_kl)
    torch.cuda.synchronize()
    rows = torch.tensor(sorted({0, 1, 777, 4095, 4096, 8191, 12345, 16383} |
                               set(np.random.default_rng(7).integers(0, cfg.N, 40).tolist())), device=DEV)
    z = f64(g["logits"][rows])
    idx = g["teacher_idx"][rows].cpu().numpy()
    lp = f64(g["teacher_logp"][rows])
    _, dl_ref, row_ref = (orc.distill_kl if mode == cb.KL_TOPK else orc.distill_kl_rest_bucket)(z, idx, lp, cfg.scale)
    e_dl = rel_err(f64(dl[rows]), dl_ref)
    e_row = rel_err(f64(row_kl[rows]), row_ref)
    print("cfg4", {"dl": e_dl, "row_kl": e_row}, flush=True)
    assert e_dl <= TOL and e_row <= 1e-4
    # the recorded tokens carry the only negative gradients of a row, exactly at teacher_idx
    neg = (dl[rows].float() < 0).cpu()
    assert torch.equal(neg, torch.tensor(dl_ref < 0))
    # every row's value and the scalar against the oracle, run in chunks of rows (a stripe of
    # 2048 rows for the rest-bucket reading, whose oracle is several times slower)
    n_rows = cfg.N if mode == cb.KL_TOPK else 2048
    fn = orc.distill_kl if mode == cb.KL_TOPK else orc.distill_kl_rest_bucket
    idx_all = g["teacher_idx"].cpu().numpy()
    lp_all = f64(g["teacher_logp"])
    chunk = 256

    def rows_of(c0):
        zc = f64(g["logits"][c0:c0 + chunk])
        return fn(zc, idx_all[c0:c0 + chunk], lp_all[c0:c0 + chunk], 1.0)[2]

    with ThreadPoolExecutor(max_workers=8) as ex:
        parts = list(ex.map(rows_of, range(0, n_rows, chunk)))
    row_all = np.concatenate(parts)
    print("cfg4 oracle rows done:", n_rows, flush=True)
    e_rows = rel_err(f64(row_kl[:n_rows]), row_all)
    assert e_rows <= 1e-4, e_rows
    if n_rows == cfg.N:
        loss_ref = cfg.scale * float(row_all.sum())
        print("cfg4 loss", loss.item(), "oracle", loss_ref, "row_kl err", e_rows, flush=True)
        assert abs(loss.item() - loss_ref) <= 1e-4 * abs(loss_ref)
    # scalar = scale * sum of the per-row values (fixed-order fp64 reduce in the library)
    expect = cfg.scale * float(row_kl.double().sum().item())
    assert abs(loss.item() - expect) <= 1e-6 * abs(expect)
    # in place (d_logits aliases logits): same bits
    buf = g["logits"].clone()
    loss2, dl2 = cb.cart_distill_kl_fwd_bwd(buf, g["teacher_idx"], g["teacher_logp"], cfg.scale, mode=mode, d_logits=buf)
    torch.cuda.synchronize()
    assert torch.equal(dl2[rows], dl[rows]) and torch.equal(dl2[::97], dl[::97]) and loss2.item() == loss.item()


@pytest.mark.parametrize("name,reqs", [("cfg5", [0, 1, 17, 63, 64, 100, 127]), ("cfg5_long", [0, 5])])
def test_decode_full_size_sampled_requests(name, reqs):
    cfg = synth.DECODE_CONFIGS[name]
    print("case", name, flush=True)
    g = synth.decode_inputs(cfg, DEV)
    o, lse = cb.cart_decode(g["q"], g["z_k"], g["z_v"], g["k_own"], g["v_own"], g["cu_lens"], cfg.max_len)
    torch.cuda.synchronize()
    cu = g["cu_lens"].cpu().numpy()
    zk, zv = f64(g["z_k"]), f64(g["z_v"])
    worst = 0.0
    for b in reqs:
        lo, hi = int(cu[b]), int(cu[b + 1])
        o_ref, l_ref = orc.decode(f64(g["q"][b:b + 1]), zk, zv, f64(g["k_own"][lo:hi]), f64(g["v_own"][lo:hi]),
                                  np.array([0, hi - lo]))
        e = max(rel_err(f64(o[b:b + 1]), o_ref), rel_err(f64(lse[b:b + 1]), l_ref))
        worst = max(worst, e)
    print(name, "worst", worst, flush=True)
    assert worst <= TOL
    assert torch.isfinite(o.float()).all() and torch.isfinite(lse).all()


def test_decode_composed_full_size_sampled_requests():
    """cfg5's shape with the cartridge in three unequal shared segments plus a 2048-slot cartridge
    of its own for every other request."""
    cfg = synth.DECODE_CONFIGS["cfg5"]
    print("case cfg5 composed", flush=True)
    g = synth.decode_inputs(cfg, DEV)
    cuts = [0, 3000, 3064, cfg.P]
    shared = [(g["z_k"][:, a:b].contiguous(), g["z_v"][:, a:b].contiguous()) for a, b in zip(cuts[:-1], cuts[1:])]
    gen = torch.Generator(device=DEV).manual_seed(5)
    n_pool, pool_p = 16, 2048
    pool_k = (0.02 * torch.randn(n_pool, cfg.Hkv, pool_p, cfg.D, generator=gen, device=DEV)).to(torch.bfloat16)
    pool_v = (0.5 * torch.randn(n_pool, cfg.Hkv, pool_p, cfg.D, generator=gen, device=DEV)).to(torch.bfloat16)
    cart_id = (torch.arange(cfg.B, device=DEV) % (2 * n_pool)).to(torch.int32)
    cart_id[cart_id >= n_pool] = -1
    o, lse = cb.cart_decode_composed(g["q"], shared, pool_k, pool_v, cart_id, g["k_own"], g["v_own"], g["cu_lens"],
                                     cfg.max_len)
    torch.cuda.synchronize()
    cu = g["cu_lens"].cpu().numpy()
    ids = cart_id.cpu().numpy()
    worst = 0.0
    for b in [0, 1, 15, 16, 17, 63, 127]:
        lo, hi = int(cu[b]), int(cu[b + 1])
        o_ref, l_ref = orc.decode_composed(f64(g["q"][b:b + 1]), [(f64(a), f64(c)) for a, c in shared], f64(pool_k),
                                           f64(pool_v), ids[b:b + 1], f64(g["k_own"][lo:hi]), f64(g["v_own"][lo:hi]),
                                           np.array([0, hi - lo]))
        worst = max(worst, rel_err(f64(o[b:b + 1]), o_ref), rel_err(f64(lse[b:b + 1]), l_ref))
    print("cfg5 composed worst", worst, flush=True)
    assert worst <= TOL
    assert torch.isfinite(o.float()).all() and torch.isfinite(lse).all()


def test_attention_packed_full_shape_one_kv_group():
    """One global batch of 64 ragged conversations at the Llama-8B layer shape: the oracle redoes
    one whole KV group (every sequence), which fixes every output of that group, dZ included."""
    cfg = synth.PACKED_CONFIGS["cfg3_packed"]
    a = synth.ATTN_CONFIGS[cfg.base]
    hk = 6
    print("case", cfg.name, "kv head", hk, flush=True)
    g = synth.attn_packed_inputs(cfg, DEV)
    ml = int(synth.packed_lengths(cfg).max())
    args = (g["q"], g["k_own"], g["v_own"], g["z_k"], g["z_v"], g["cu_seqlens"], ml)
    o, lse = cb.cart_attn_varlen_fwd(*args)
    dq, dk, dv, dzk, dzv = cb.cart_attn_varlen_bwd(*args, o, lse, g["d_o"])
    torch.cuda.synchronize()
    G = a.Hq // a.Hkv
    hs = slice(hk * G, (hk + 1) * G)
    cu = g["cu_seqlens"].cpu().numpy()
    q, do = f64(g["q"][:, hs]), f64(g["d_o"][:, hs])
    k, v = f64(g["k_own"][:, hk:hk + 1]), f64(g["v_own"][:, hk:hk + 1])
    zk, zv = f64(g["z_k"][hk:hk + 1]), f64(g["z_v"][hk:hk + 1])
    o_ref, lse_ref = orc.attn_varlen_fwd(q, k, v, zk, zv, cu)
    r = orc.attn_varlen_bwd(q, k, v, zk, zv, do, cu)
    errs = {
        "o": rel_err(f64(o[:, hs]), o_ref), "lse": rel_err(f64(lse[hs]), lse_ref),
        "dq": rel_err(f64(dq[:, hs]), r[0]), "dk": rel_err(f64(dk[:, hk:hk + 1]), r[1]),
        "dv": rel_err(f64(dv[:, hk:hk + 1]), r[2]), "dzk": rel_err(f64(dzk[hk:hk + 1]), r[3]),
        "dzv": rel_err(f64(dzv[hk:hk + 1]), r[4]),
    }
    print(cfg.name, errs, flush=True)
    for kk, e in errs.items():
        assert e <= TOL, (cfg.name, kk, e)
    again = cb.cart_attn_varlen_bwd(*args, o, lse, g["d_o"])
    torch.cuda.synchronize()
    for x, y in zip((dq, dk, dv, dzk, dzv), again):
        assert torch.equal(x, y)
