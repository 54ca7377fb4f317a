"""Pins for the attention oracle (forward and backward).  CPU only.

Nothing here re-types the oracle's vectorised formula: the comparisons are a scalar-loop
evaluation of Eq. 1 written independently below, hand-worked numbers, closed forms,
structural identities and central finite differences.
"""
import json
import math
import os

import numpy as np
import pytest

from oracle import cartridge_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------------------------------------
# independent references written for the tests only
# ---------------------------------------------------------------------------------------------
def textbook_causal(q, k, v, scale):
    """Eq. 1 literally, one head: y[i] = sum_{j<=i} exp(q_i.k_j*scale) v_j / sum_{t<=i} exp(...)."""
    n, d = q.shape
    y = np.zeros((n, v.shape[1]))
    lse = np.zeros(n)
    for i in range(n):
        num = np.zeros(v.shape[1])
        den = 0.0
        for j in range(i + 1):
            w = math.exp(sum(q[i, c] * k[j, c] for c in range(d)) * scale)
            num += w * v[j]
            den += w
        y[i] = num / den
        lse[i] = math.log(den)
    return y, lse


def brute_cartridge(q, k_own, v_own, z_k, z_v, scale):
    """Scalar loops over the cartridge cache: prefix slots always visible, own keys j <= i."""
    B, S, Hq, d = q.shape
    Hkv, p, _ = z_k.shape
    G = Hq // Hkv
    o = np.zeros((B, S, Hq, d))
    lse = np.zeros((B, Hq, S))
    for b in range(B):
        for h in range(Hq):
            hk = h // G
            for i in range(S):
                ws, vs = [], []
                for t in range(p):
                    ws.append(math.exp(scale * float(np.dot(q[b, i, h], z_k[hk, t]))))
                    vs.append(z_v[hk, t])
                for j in range(i + 1):
                    ws.append(math.exp(scale * float(np.dot(q[b, i, h], k_own[b, j, hk]))))
                    vs.append(v_own[b, j, hk])
                den = sum(ws)
                o[b, i, h] = sum(w * v for w, v in zip(ws, vs)) / den
                lse[b, h, i] = math.log(den)
    return o, lse


def rand_problem(rng, B, S, Hq, Hkv, d, p, std=1.0):
    return dict(
        q=rng.normal(0, std, (B, S, Hq, d)),
        k_own=rng.normal(0, std, (B, S, Hkv, d)),
        v_own=rng.normal(0, 1, (B, S, Hkv, d)),
        z_k=rng.normal(0, std, (Hkv, p, d)),
        z_v=rng.normal(0, 1, (Hkv, p, d)),
    )


# ---------------------------------------------------------------------------------------------
# forward
# ---------------------------------------------------------------------------------------------
def test_hand_worked_example():
    with open(os.path.join(GOLDEN, "attn_worked_example.json")) as f:
        g = json.load(f)
    q = np.log(np.array(g["q_ln_of"])).reshape(1, 2, 1, 1)
    k = np.array(g["k_own"]).reshape(1, 2, 1, 1)
    v = np.array(g["v_own"]).reshape(1, 2, 1, 1)
    zk = np.array(g["z_k"]).reshape(1, 1, 1)
    zv = np.array(g["z_v"]).reshape(1, 1, 1)
    o, lse = orc.attn_fwd(q, k, v, zk, zv, scale=g["scale"])
    np.testing.assert_allclose(o.ravel(), g["o"], rtol=1e-13)
    np.testing.assert_allclose(lse.ravel(), np.log(g["lse_ln_of"]), rtol=1e-13)


def test_p0_is_textbook_causal_attention():
    rng = np.random.default_rng(1)
    pr = rand_problem(rng, 2, 9, 2, 2, 5, 0)
    scale = 1.0 / math.sqrt(5)
    o, lse = orc.attn_fwd(**pr)
    for b in range(2):
        for h in range(2):
            y, l = textbook_causal(pr["q"][b, :, h], pr["k_own"][b, :, h], pr["v_own"][b, :, h], scale)
            np.testing.assert_allclose(o[b, :, h], y, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(lse[b, h], l, rtol=1e-12, atol=1e-13)


def test_brute_force_tiny_with_prefix_and_gqa():
    rng = np.random.default_rng(2)
    for (B, S, Hq, Hkv, d, p) in [(1, 4, 1, 1, 2, 2), (2, 3, 4, 2, 3, 1), (1, 5, 6, 2, 2, 3)]:
        pr = rand_problem(rng, B, S, Hq, Hkv, d, p)
        o, lse = orc.attn_fwd(**pr, scale=0.7)
        ob, lb = brute_cartridge(**pr, scale=0.7)
        np.testing.assert_allclose(o, ob, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(lse, lb, rtol=1e-12, atol=1e-13)


def test_concatenation_identity():
    """Cartridge attention == the last S rows of plain causal attention over [Z ; own]."""
    rng = np.random.default_rng(3)
    B, S, H, d, p = 2, 7, 1, 4, 5
    pr = rand_problem(rng, B, S, H, H, d, p)
    o, lse = orc.attn_fwd(**pr)
    scale = 1.0 / math.sqrt(d)
    for b in range(B):
        kk = np.concatenate([pr["z_k"][0], pr["k_own"][b, :, 0]])
        vv = np.concatenate([pr["z_v"][0], pr["v_own"][b, :, 0]])
        qq = np.concatenate([rng.normal(size=(p, d)), pr["q"][b, :, 0]])   # first p queries arbitrary
        y, l = textbook_causal(qq, kk, vv, scale)
        np.testing.assert_allclose(o[b, :, 0], y[p:], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(lse[b, 0], l[p:], rtol=1e-12, atol=1e-13)


def test_softmax_rows_sum_to_one():
    """With every value vector equal to the all-ones vector the output is exactly one, and
    exp(score - lse) summed over the visible keys is one."""
    rng = np.random.default_rng(4)
    B, S, Hq, Hkv, d, p = 2, 11, 4, 2, 6, 7
    pr = rand_problem(rng, B, S, Hq, Hkv, d, p, std=2.0)
    pr["v_own"] = np.ones_like(pr["v_own"])
    pr["z_v"] = np.ones_like(pr["z_v"])
    o, lse = orc.attn_fwd(**pr)
    assert np.abs(o - 1.0).max() < 1e-12
    scale = 1.0 / math.sqrt(d)
    for b in range(B):
        for h in range(Hq):
            hk = h // (Hq // Hkv)
            for i in range(S):
                tot = sum(math.exp(scale * pr["q"][b, i, h] @ pr["z_k"][hk, t] - lse[b, h, i]) for t in range(p))
                tot += sum(math.exp(scale * pr["q"][b, i, h] @ pr["k_own"][b, j, hk] - lse[b, h, i])
                           for j in range(i + 1))
                assert abs(tot - 1.0) < 1e-12


def test_equal_keys_give_mean_of_visible_values():
    rng = np.random.default_rng(5)
    B, S, H, d, p = 1, 6, 1, 3, 4
    pr = rand_problem(rng, B, S, H, H, d, p)
    kvec = rng.normal(size=d)
    pr["k_own"][:] = kvec
    pr["z_k"][:] = kvec
    o, lse = orc.attn_fwd(**pr)
    allv = np.concatenate([pr["z_v"][0], pr["v_own"][0, :, 0]])
    scale = 1.0 / math.sqrt(d)
    for i in range(S):
        np.testing.assert_allclose(o[0, i, 0], allv[: p + i + 1].mean(axis=0), rtol=1e-12)
        s = scale * pr["q"][0, i, 0] @ kvec
        assert abs(lse[0, 0, i] - (s + math.log(p + i + 1))) < 1e-12


def test_score_shift_and_scale_argument():
    rng = np.random.default_rng(6)
    pr = rand_problem(rng, 1, 5, 2, 1, 4, 3)
    o, lse = orc.attn_fwd(**pr, scale=0.5)
    # scale can be folded into q
    pr2 = dict(pr, q=0.5 * pr["q"])
    o2, lse2 = orc.attn_fwd(**pr2, scale=1.0)
    np.testing.assert_allclose(o, o2, rtol=1e-12)
    np.testing.assert_allclose(lse, lse2, rtol=1e-12)
    # one extra feature equal to 1 in q and to c in every key adds scale*c to every score
    c = 1.7
    q3 = np.concatenate([pr["q"], np.ones(pr["q"].shape[:-1] + (1,))], axis=-1)
    k3 = np.concatenate([pr["k_own"], c * np.ones(pr["k_own"].shape[:-1] + (1,))], axis=-1)
    zk3 = np.concatenate([pr["z_k"], c * np.ones(pr["z_k"].shape[:-1] + (1,))], axis=-1)
    v3 = np.concatenate([pr["v_own"], np.zeros(pr["v_own"].shape[:-1] + (1,))], axis=-1)
    zv3 = np.concatenate([pr["z_v"], np.zeros(pr["z_v"].shape[:-1] + (1,))], axis=-1)
    o3, lse3 = orc.attn_fwd(q3, k3, v3, zk3, zv3, scale=0.5)
    np.testing.assert_allclose(o3[..., :-1], o, rtol=1e-12)
    np.testing.assert_allclose(lse3, lse + 0.5 * c, rtol=1e-12)


def test_gqa_equals_mha_with_repeated_kv_heads():
    rng = np.random.default_rng(7)
    B, S, Hq, Hkv, d, p = 2, 6, 6, 2, 4, 3
    G = Hq // Hkv
    pr = rand_problem(rng, B, S, Hq, Hkv, d, p)
    o, lse = orc.attn_fwd(**pr)
    rep = dict(pr, k_own=np.repeat(pr["k_own"], G, axis=2), v_own=np.repeat(pr["v_own"], G, axis=2),
               z_k=np.repeat(pr["z_k"], G, axis=0), z_v=np.repeat(pr["z_v"], G, axis=0))
    o2, lse2 = orc.attn_fwd(**rep)
    np.testing.assert_allclose(o, o2, rtol=1e-13)
    np.testing.assert_allclose(lse, lse2, rtol=1e-13)


def test_future_own_tokens_do_not_matter_but_prefix_does():
    rng = np.random.default_rng(8)
    pr = rand_problem(rng, 1, 6, 1, 1, 3, 2)
    o, _ = orc.attn_fwd(**pr)
    pr2 = {k: v.copy() for k, v in pr.items()}
    pr2["k_own"][0, 4:] += 5.0
    pr2["v_own"][0, 4:] -= 3.0
    o2, _ = orc.attn_fwd(**pr2)
    np.testing.assert_array_equal(o[0, :4], o2[0, :4])
    assert np.abs(o[0, 4:] - o2[0, 4:]).max() > 1e-3
    pr3 = {k: v.copy() for k, v in pr.items()}
    pr3["z_v"][0, 1] += 1.0
    o3, _ = orc.attn_fwd(**pr3)
    assert np.abs(o3 - o).min() > 0          # every row sees every prefix slot


# ---------------------------------------------------------------------------------------------
# backward
# ---------------------------------------------------------------------------------------------
def _objective(pr, d_o, scale):
    o, _ = orc.attn_fwd(**pr, scale=scale)
    return float((o * d_o).sum())


@pytest.mark.parametrize("shape", [(2, 5, 4, 2, 3, 3), (1, 4, 2, 2, 2, 0), (2, 3, 3, 1, 4, 5)])
def test_finite_differences(shape):
    B, S, Hq, Hkv, d, p = shape
    rng = np.random.default_rng(10 + p)
    pr = rand_problem(rng, B, S, Hq, Hkv, d, p)
    d_o = rng.normal(size=(B, S, Hq, d))
    scale = 0.6
    grads = orc.attn_bwd(**pr, d_o=d_o, scale=scale)
    names = ["q", "k_own", "v_own", "z_k", "z_v"]
    eps = 1e-5
    for name, g in zip(names, grads):
        x = pr[name]
        assert g.shape == x.shape
        num = np.zeros_like(x)
        for ix in np.ndindex(*x.shape):
            old = x[ix]
            x[ix] = old + eps
            fp = _objective(pr, d_o, scale)
            x[ix] = old - eps
            fm = _objective(pr, d_o, scale)
            x[ix] = old
            num[ix] = (fp - fm) / (2 * eps)
        if x.size:
            err = np.abs(num - g).max() / max(np.abs(num).max(), 1e-30)
            assert err < 1e-6, (name, err)


def test_dz_is_sum_over_batch():
    rng = np.random.default_rng(20)
    B, S, Hq, Hkv, d, p = 3, 5, 4, 2, 3, 4
    pr = rand_problem(rng, B, S, Hq, Hkv, d, p)
    d_o = rng.normal(size=(B, S, Hq, d))
    full = orc.attn_bwd(**pr, d_o=d_o)
    acc_k = np.zeros_like(full[3])
    acc_v = np.zeros_like(full[4])
    for b in range(B):
        one = {k: (v[b:b + 1] if k in ("q", "k_own", "v_own") else v) for k, v in pr.items()}
        g = orc.attn_bwd(**one, d_o=d_o[b:b + 1])
        acc_k += g[3]
        acc_v += g[4]
        np.testing.assert_allclose(g[0][0], full[0][b], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(g[1][0], full[1][b], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(acc_k, full[3], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(acc_v, full[4], rtol=1e-12, atol=1e-14)


def test_dz_matches_concatenated_plain_attention():
    """Treat [Z ; own] as one plain causal sequence (p = 0 path) whose first p query rows get a
    zero upstream gradient: its dK/dV rows 0..p-1, summed over the batch, are dZ_k/dZ_v."""
    rng = np.random.default_rng(21)
    B, S, H, d, p = 2, 5, 1, 3, 4
    pr = rand_problem(rng, B, S, H, H, d, p)
    d_o = rng.normal(size=(B, S, H, d))
    g = orc.attn_bwd(**pr, d_o=d_o)
    acc_k = np.zeros((p, d))
    acc_v = np.zeros((p, d))
    empty = np.zeros((H, 0, d))
    for b in range(B):
        qq = np.concatenate([rng.normal(size=(p, d)), pr["q"][b, :, 0]])[None, :, None, :]
        kk = np.concatenate([pr["z_k"][0], pr["k_own"][b, :, 0]])[None, :, None, :]
        vv = np.concatenate([pr["z_v"][0], pr["v_own"][b, :, 0]])[None, :, None, :]
        dd = np.concatenate([np.zeros((p, d)), d_o[b, :, 0]])[None, :, None, :]
        gc = orc.attn_bwd(qq, kk, vv, empty, empty, dd)
        acc_k += gc[1][0, :p, 0]
        acc_v += gc[2][0, :p, 0]
        np.testing.assert_allclose(gc[1][0, p:, 0], g[1][b, :, 0], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(gc[0][0, p:, 0], g[0][b, :, 0], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(acc_k, g[3][0], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(acc_v, g[4][0], rtol=1e-11, atol=1e-13)


def test_key_gradients_sum_to_zero():
    """Adding one vector to every key of a KV head shifts each score row by a constant, which the
    softmax ignores; so the key gradients of that head (prefix + own, all sequences) sum to 0."""
    rng = np.random.default_rng(22)
    B, S, Hq, Hkv, d, p = 2, 6, 4, 2, 3, 3
    pr = rand_problem(rng, B, S, Hq, Hkv, d, p)
    d_o = rng.normal(size=(B, S, Hq, d))
    _, dk, _, dzk, _ = orc.attn_bwd(**pr, d_o=d_o)
    tot = dk.sum(axis=(0, 1)) + dzk.sum(axis=1)
    assert np.abs(tot).max() < 1e-12 * max(1.0, np.abs(dk).max())


def test_value_gradient_closed_form_for_uniform_attention():
    """q = 0 makes every visible weight 1/(p+i+1): dV_j = sum_{i>=j} dO_i/(p+i+1) and
    dZ_v[t] = sum_b sum_i dO_i/(p+i+1)."""
    rng = np.random.default_rng(23)
    B, S, H, d, p = 2, 5, 1, 2, 3
    pr = rand_problem(rng, B, S, H, H, d, p)
    pr["q"][:] = 0.0
    d_o = rng.normal(size=(B, S, H, d))
    _, _, dv, _, dzv = orc.attn_bwd(**pr, d_o=d_o)
    w = 1.0 / (p + np.arange(S) + 1.0)
    for b in range(B):
        for j in range(S):
            np.testing.assert_allclose(dv[b, j, 0], (d_o[b, j:, 0] * w[j:, None]).sum(0), rtol=1e-12)
    exp_z = sum((d_o[b, :, 0] * w[:, None]).sum(0) for b in range(B))
    for t in range(p):
        np.testing.assert_allclose(dzv[0, t], exp_z, rtol=1e-12)
