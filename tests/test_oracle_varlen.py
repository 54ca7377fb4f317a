"""Pins for the packed variable-length attention oracle."""
import numpy as np
import pytest

from oracle import cartridge_oracle as orc


def _case(seed, lens, Hq=4, Hkv=2, d=8, p=5):
    rng = np.random.default_rng(seed)
    cu = np.concatenate([[0], np.cumsum(lens)])
    T = int(cu[-1])
    return dict(q=rng.normal(size=(T, Hq, d)), k=rng.normal(size=(T, Hkv, d)), v=rng.normal(size=(T, Hkv, d)),
                zk=rng.normal(size=(Hkv, p, d)), zv=rng.normal(size=(Hkv, p, d)), do=rng.normal(size=(T, Hq, d)), cu=cu)


def test_equal_lengths_are_the_batched_functions():
    c = _case(1, [6, 6, 6])
    B, S = 3, 6
    o, lse = orc.attn_varlen_fwd(c["q"], c["k"], c["v"], c["zk"], c["zv"], c["cu"])
    rs = lambda x: x.reshape(B, S, *x.shape[1:])
    o2, lse2 = orc.attn_fwd(rs(c["q"]), rs(c["k"]), rs(c["v"]), c["zk"], c["zv"])
    np.testing.assert_allclose(o, o2.reshape(o.shape), atol=1e-14)
    np.testing.assert_allclose(lse, np.transpose(lse2, (1, 0, 2)).reshape(lse.shape), atol=1e-14)
    g = orc.attn_varlen_bwd(c["q"], c["k"], c["v"], c["zk"], c["zv"], c["do"], c["cu"])
    g2 = orc.attn_bwd(rs(c["q"]), rs(c["k"]), rs(c["v"]), c["zk"], c["zv"], rs(c["do"]))
    for a, b in zip(g[:3], g2[:3]):
        np.testing.assert_allclose(a, b.reshape(a.shape), atol=1e-13)
    np.testing.assert_allclose(g[3], g2[3], atol=1e-13)
    np.testing.assert_allclose(g[4], g2[4], atol=1e-13)


def test_sequences_do_not_see_each_other_and_a_one_token_sequence():
    c = _case(2, [3, 1, 5])
    o, lse = orc.attn_varlen_fwd(c["q"], c["k"], c["v"], c["zk"], c["zv"], c["cu"])
    # changing sequence 2's keys leaves sequences 0 and 1 alone
    k2 = c["k"].copy()
    k2[4:] += 1.0
    o2, _ = orc.attn_varlen_fwd(c["q"], k2, c["v"], c["zk"], c["zv"], c["cu"])
    np.testing.assert_array_equal(o[:4], o2[:4])
    assert np.abs(o[4:] - o2[4:]).max() > 1e-3
    # the one-token sequence (row 3): softmax over the prefix and its own key, written out
    d = c["q"].shape[-1]
    for h in range(4):
        hk = h // 2
        keys = np.concatenate([c["zk"][hk], c["k"][3:4, hk]])
        vals = np.concatenate([c["zv"][hk], c["v"][3:4, hk]])
        s = keys @ c["q"][3, h] / np.sqrt(d)
        w = np.exp(s - s.max()); w /= w.sum()
        np.testing.assert_allclose(o[3, h], w @ vals, atol=1e-14)


def test_gradient_finite_differences_and_prefix_gradient_adds_over_sequences():
    c = _case(3, [2, 4])
    g = orc.attn_varlen_bwd(c["q"], c["k"], c["v"], c["zk"], c["zv"], c["do"], c["cu"])
    f = lambda **kw: (orc.attn_varlen_fwd(kw.get("q", c["q"]), kw.get("k", c["k"]), kw.get("v", c["v"]),
                                         kw.get("zk", c["zk"]), kw.get("zv", c["zv"]), c["cu"])[0] * c["do"]).sum()
    h = 1e-6
    for name, gi, pos in [("q", 0, (5, 1, 3)), ("k", 1, (0, 1, 2)), ("v", 2, (3, 0, 7)), ("zk", 3, (1, 4, 0)), ("zv", 4, (0, 2, 5))]:
        xp, xm = c[name].copy(), c[name].copy()
        xp[pos] += h
        xm[pos] -= h
        fd = (f(**{name: xp}) - f(**{name: xm})) / (2 * h)
        assert fd == pytest.approx(g[gi][pos], abs=1e-7)
    # d_z of the packed batch = sum of the d_z of its sequences run alone
    parts = [orc.attn_varlen_bwd(c["q"][a:b], c["k"][a:b], c["v"][a:b], c["zk"], c["zv"], c["do"][a:b], [0, b - a])
             for a, b in zip(c["cu"][:-1], c["cu"][1:])]
    np.testing.assert_allclose(g[3], sum(p[3] for p in parts), atol=1e-13)
    np.testing.assert_allclose(g[4], sum(p[4] for p in parts), atol=1e-13)
