"""Pins for the composed-cartridge decode oracle (Sec. 5.4 composition; per-request cartridges)."""
import numpy as np
import pytest
from scipy.special import logsumexp

from oracle import cartridge_oracle as orc


def _case(seed, B=5, Hq=4, Hkv=2, d=8, ps=(3, 5, 2), n_pool=3, pc=4):
    rng = np.random.default_rng(seed)
    lens = rng.integers(1, 6, size=B)
    cu = np.concatenate([[0], np.cumsum(lens)])
    T = int(cu[-1])
    shared = [(rng.normal(size=(Hkv, p, d)), rng.normal(size=(Hkv, p, d))) for p in ps]
    return dict(q=rng.normal(size=(B, Hq, d)), shared=shared, pool_k=rng.normal(size=(n_pool, Hkv, pc, d)),
                pool_v=rng.normal(size=(n_pool, Hkv, pc, d)), cart_id=rng.integers(-1, n_pool, size=B),
                k_own=rng.normal(size=(T, Hkv, d)), v_own=rng.normal(size=(T, Hkv, d)), cu=cu)


def test_shared_segments_equal_one_concatenated_cartridge_in_any_order():
    c = _case(1)
    o, lse = orc.decode_composed(c["q"], c["shared"], None, None, None, c["k_own"], c["v_own"], c["cu"])
    zk = np.concatenate([a for a, _ in c["shared"]], axis=1)
    zv = np.concatenate([b for _, b in c["shared"]], axis=1)
    o1, lse1 = orc.decode(c["q"], zk, zv, c["k_own"], c["v_own"], c["cu"])
    np.testing.assert_allclose(o, o1, atol=1e-13)
    np.testing.assert_allclose(lse, lse1, atol=1e-13)
    # attention over a set of keys: the order of the segments does not matter
    o2, lse2 = orc.decode_composed(c["q"], c["shared"][::-1], None, None, None, c["k_own"], c["v_own"], c["cu"])
    np.testing.assert_allclose(o2, o, atol=1e-13)
    np.testing.assert_allclose(lse2, lse, atol=1e-13)


def test_private_cartridge_is_an_extra_segment_of_that_request_only():
    c = _case(2)
    o, lse = orc.decode_composed(c["q"], c["shared"], c["pool_k"], c["pool_v"], c["cart_id"], c["k_own"],
                                 c["v_own"], c["cu"])
    for b in range(c["q"].shape[0]):
        segs = list(c["shared"])
        if c["cart_id"][b] >= 0:
            segs.append((c["pool_k"][c["cart_id"][b]], c["pool_v"][c["cart_id"][b]]))
        sl = slice(c["cu"][b], c["cu"][b + 1])
        ob, lb = orc.decode_composed(c["q"][b:b + 1], segs, None, None, None, c["k_own"][sl], c["v_own"][sl],
                                     np.array([0, sl.stop - sl.start]))
        np.testing.assert_allclose(o[b], ob[0], atol=1e-13)
        np.testing.assert_allclose(lse[b], lb[0], atol=1e-13)
    # the same private cartridge for every request is a shared segment
    ids = np.full(c["q"].shape[0], 1)
    o3, l3 = orc.decode_composed(c["q"], c["shared"], c["pool_k"], c["pool_v"], ids, c["k_own"], c["v_own"], c["cu"])
    o4, l4 = orc.decode_composed(c["q"], c["shared"] + [(c["pool_k"][1], c["pool_v"][1])], None, None, None,
                                 c["k_own"], c["v_own"], c["cu"])
    np.testing.assert_allclose(o3, o4, atol=1e-13)
    np.testing.assert_allclose(l3, l4, atol=1e-13)


def test_parts_merge_by_their_log_sum_exps():
    """Softmax over a union of key sets = lse-weighted mix of the softmaxes over the parts,
    each part evaluated as an attention of its own (own rows as the only keys: p = 0 decode)."""
    c = _case(3, ps=(4, 6))
    B, Hq, d = c["q"].shape
    Hkv = c["k_own"].shape[1]
    o, lse = orc.decode_composed(c["q"], c["shared"], None, None, None, c["k_own"], c["v_own"], c["cu"])
    parts = []
    for zk, zv in c["shared"]:
        # a part alone: its slots as "own rows" of every request, no prefix at all
        p = zk.shape[1]
        k_rep = np.concatenate([np.transpose(zk, (1, 0, 2))] * B, axis=0)
        v_rep = np.concatenate([np.transpose(zv, (1, 0, 2))] * B, axis=0)
        parts.append(orc.decode(c["q"], np.zeros((Hkv, 0, d)), np.zeros((Hkv, 0, d)), k_rep, v_rep,
                                np.arange(B + 1) * p))
    parts.append(orc.decode(c["q"], np.zeros((Hkv, 0, d)), np.zeros((Hkv, 0, d)), c["k_own"], c["v_own"], c["cu"]))
    ls = np.stack([l for _, l in parts])
    tot = logsumexp(ls, axis=0)
    mix = sum(np.exp(l - tot)[..., None] * oo for oo, l in parts)
    np.testing.assert_allclose(lse, tot, atol=1e-12)
    np.testing.assert_allclose(o, mix, atol=1e-12)


def test_one_dominant_key_and_uniform_keys():
    rng = np.random.default_rng(4)
    Hkv, d = 1, 4
    q = np.array([[[2.0, 0, 0, 0]]])
    zk1 = np.zeros((Hkv, 3, d)); zv1 = rng.normal(size=(Hkv, 3, d))
    zk2 = np.zeros((Hkv, 2, d)); zv2 = rng.normal(size=(Hkv, 2, d))
    k_own = np.zeros((1, Hkv, d)); v_own = rng.normal(size=(1, Hkv, d))
    o, lse = orc.decode_composed(q, [(zk1, zv1), (zk2, zv2)], None, None, None, k_own, v_own, [0, 1])
    allv = np.concatenate([zv1[0], zv2[0], v_own[:, 0]])
    np.testing.assert_allclose(o[0, 0], allv.mean(axis=0), atol=1e-14)     # equal scores: the mean
    assert lse[0, 0] == pytest.approx(np.log(6.0))
    zk2[0, 1, 0] = 400.0                                                   # one key takes all the mass
    o, lse = orc.decode_composed(q, [(zk1, zv1), (zk2, zv2)], None, None, None, k_own, v_own, [0, 1])
    np.testing.assert_allclose(o[0, 0], zv2[0, 1], atol=1e-12)
    assert lse[0, 0] == pytest.approx(400.0 * 2.0 / 2.0)                   # scale = 1/sqrt(4)
