"""Pins for the two further loss modes of the oracle: the rest-bucket KL and next-token
cross-entropy (Sec. 4.2 / 5.3: the objective context distillation is compared with)."""
import math

import numpy as np
import pytest
from scipy.special import log_softmax, rel_entr, softmax

from oracle import cartridge_oracle as orc


def _teacher(rng, n, v, k, mass):
    idx = np.stack([rng.choice(v, size=k, replace=False) for _ in range(n)])
    w = rng.normal(size=(n, k)) * 2.0
    p = softmax(w, axis=1) * mass
    return idx, np.log(p)


def test_rest_bucket_is_the_kl_of_the_coarsened_distributions():
    """Build the (k+1)-outcome distributions explicitly and hand them to scipy's rel_entr."""
    rng = np.random.default_rng(1)
    N, V, K = 5, 40, 6
    z = rng.normal(size=(N, V)) * 2
    idx, lp = _teacher(rng, N, V, K, 0.8)
    _, _, row = orc.distill_kl_rest_bucket(z, idx, lp)
    s = softmax(z, axis=1)
    for n in range(N):
        t_c = np.append(np.exp(lp[n]), 1 - np.exp(lp[n]).sum())
        s_c = np.append(s[n, idx[n]], 1 - s[n, idx[n]].sum())
        assert row[n] == pytest.approx(rel_entr(t_c, s_c).sum(), rel=1e-12)
        assert row[n] >= 0


def test_rest_bucket_full_mass_equals_truncated_reading_and_full_teacher_is_textbook_kl():
    rng = np.random.default_rng(2)
    N, V, K = 4, 30, 5
    z = rng.normal(size=(N, V))
    idx, lp = _teacher(rng, N, V, K, 1.0)
    a = orc.distill_kl(z, idx, lp, 0.5)
    d = orc.distill_kl_rest_bucket(z, idx, lp, 0.5)
    assert d[0] == pytest.approx(a[0], rel=1e-12)
    np.testing.assert_allclose(d[1], a[1], rtol=0, atol=1e-14)
    # k = V: the teacher is a full distribution
    idx_full = np.tile(np.arange(V), (N, 1))
    t = softmax(rng.normal(size=(N, V)), axis=1)
    loss, g, row = orc.distill_kl_rest_bucket(z, idx_full, np.log(t))
    np.testing.assert_allclose(row, rel_entr(t, softmax(z, axis=1)).sum(axis=1), rtol=1e-12)
    np.testing.assert_allclose(g, softmax(z, axis=1) - t, atol=1e-14)


@pytest.mark.parametrize("mass", [0.6, 0.95])
def test_rest_bucket_vanishes_exactly_when_student_matches_teacher_on_the_support(mass):
    """Unlike the truncated reading (zero gradient at s = t / M), the minimum sits at s = t."""
    rng = np.random.default_rng(3)
    V, K = 25, 4
    idx, lp = _teacher(rng, 1, V, K, mass)
    # student: t on the support, the remaining 1 - M spread unevenly over the other tokens
    s = np.zeros(V)
    s[idx[0]] = np.exp(lp[0])
    off = np.setdiff1d(np.arange(V), idx[0])
    w = rng.random(off.size) + 0.1
    s[off] = (1 - mass) * w / w.sum()
    loss, g, row = orc.distill_kl_rest_bucket(np.log(s)[None, :] + 3.7, idx, lp)
    assert abs(loss) < 1e-13 and np.abs(g).max() < 1e-13
    # move mass inside the support: strictly positive
    s2 = s.copy()
    s2[idx[0][0]] *= 0.5
    s2[idx[0][1]] += 0.5 * s[idx[0][0]]
    assert orc.distill_kl_rest_bucket(np.log(s2)[None, :], idx, lp)[0] > 1e-4


def test_rest_bucket_gradient_finite_differences_rows_sum_to_zero_ignored_entries():
    rng = np.random.default_rng(4)
    N, V, K = 3, 17, 5
    z = rng.normal(size=(N, V))
    idx, lp = _teacher(rng, N, V, K, 0.7)
    idx[1, 2] = -1                      # an ignored record
    loss, g, _ = orc.distill_kl_rest_bucket(z, idx, lp, 1.3)
    np.testing.assert_allclose(g.sum(axis=1), 0, atol=1e-13)
    h = 1e-6
    for (n, v) in [(0, 0), (0, int(idx[0, 0])), (1, int(idx[1, 0])), (1, int(idx[1, 3])), (2, 9), (2, 16)]:
        zp, zm = z.copy(), z.copy()
        zp[n, v] += h
        zm[n, v] -= h
        fd = (orc.distill_kl_rest_bucket(zp, idx, lp, 1.3)[0] - orc.distill_kl_rest_bucket(zm, idx, lp, 1.3)[0]) / (2 * h)
        assert fd == pytest.approx(g[n, v], abs=1e-8)
    # dropping the ignored record from the arrays gives the same numbers
    keep = [0, 1, 3, 4]
    l1 = orc.distill_kl_rest_bucket(z[1:2], idx[1:2], lp[1:2])
    l2 = orc.distill_kl_rest_bucket(z[1:2], idx[1:2, keep], lp[1:2, keep])
    assert l1[0] == pytest.approx(l2[0], rel=1e-13)
    np.testing.assert_allclose(l1[1], l2[1], atol=1e-15)
    # shift invariance
    np.testing.assert_allclose(orc.distill_kl_rest_bucket(z + 5.0, idx, lp, 1.3)[1], g, atol=1e-13)


def test_ntp_cross_entropy_is_minus_log_softmax_at_the_label():
    rng = np.random.default_rng(5)
    N, V = 6, 23
    z = rng.normal(size=(N, V)) * 3
    lab = rng.integers(0, V, size=N)
    lab[2] = -100                        # ignored
    loss, g, row = orc.ntp_cross_entropy(z, lab, 0.25)
    ls = log_softmax(z, axis=1)
    for n in range(N):
        if lab[n] < 0:
            assert row[n] == 0 and not g[n].any()
        else:
            assert row[n] == pytest.approx(-ls[n, lab[n]], rel=1e-13)
            onehot = np.zeros(V)
            onehot[lab[n]] = 1
            np.testing.assert_allclose(g[n], 0.25 * (softmax(z[n]) - onehot), atol=1e-15)
    assert loss == pytest.approx(0.25 * row.sum(), rel=1e-14)
    # hand-worked: two logits (0, log 3) -> softmax (1/4, 3/4)
    l2, g2, _ = orc.ntp_cross_entropy(np.array([[0.0, math.log(3.0)]]), np.array([0]))
    assert l2 == pytest.approx(math.log(4.0), rel=1e-14)
    np.testing.assert_allclose(g2, [[-0.75, 0.75]], atol=1e-15)
    # finite differences
    h = 1e-6
    for (n, v) in [(0, 1), (1, int(lab[1])), (5, 22)]:
        zp, zm = z.copy(), z.copy()
        zp[n, v] += h
        zm[n, v] -= h
        fd = (orc.ntp_cross_entropy(zp, lab, 0.25)[0] - orc.ntp_cross_entropy(zm, lab, 0.25)[0]) / (2 * h)
        assert fd == pytest.approx(g[n, v], abs=1e-8)


def test_ntp_is_the_k1_unit_mass_case_of_both_distillation_readings():
    rng = np.random.default_rng(6)
    N, V = 4, 11
    z = rng.normal(size=(N, V))
    lab = np.array([3, -1, 0, 10])
    ce = orc.ntp_cross_entropy(z, lab, 2.0)
    for f in (orc.distill_kl, orc.distill_kl_rest_bucket):
        r = f(z, lab[:, None], np.zeros((N, 1)), 2.0)
        assert r[0] == pytest.approx(ce[0], rel=1e-13)
        np.testing.assert_allclose(r[1], ce[1], atol=1e-14)
