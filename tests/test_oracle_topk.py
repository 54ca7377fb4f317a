"""Pins for the teacher top-k oracle (App. A.2: top output probabilities are recorded)."""
import numpy as np
import pytest
from scipy.special import log_softmax

from oracle import cartridge_oracle as orc


def test_matches_stable_argsort_and_log_softmax():
    rng = np.random.default_rng(1)
    z = rng.normal(size=(7, 300)) * 3
    idx, lp = orc.teacher_topk(z, 20)
    ls = log_softmax(z, axis=1)
    for n in range(7):
        ref = np.argsort(-z[n], kind="stable")[:20]
        assert (idx[n] == ref).all()
        np.testing.assert_allclose(lp[n], ls[n, ref], rtol=0, atol=1e-13)
        assert (np.diff(lp[n]) <= 0).all()


def test_ties_go_to_the_lower_index_and_all_equal_rows():
    z = np.array([[1.0, 3.0, 3.0, 0.0, 3.0, 2.0, 2.0],
                  [5.0, 5.0, 5.0, 5.0, 5.0, 5.0, 5.0]])
    idx, lp = orc.teacher_topk(z, 4)
    assert idx[0].tolist() == [1, 2, 4, 5]
    assert idx[1].tolist() == [0, 1, 2, 3]
    np.testing.assert_allclose(lp[1], np.log(1 / 7), atol=1e-14)
    # hand-worked: logits (0, log 2, log 5): probabilities 1/8, 2/8, 5/8
    idx, lp = orc.teacher_topk(np.log(np.array([[1.0, 2.0, 5.0]])), 2)
    assert idx[0].tolist() == [2, 1]
    np.testing.assert_allclose(np.exp(lp[0]), [5 / 8, 2 / 8], atol=1e-15)


def test_permutation_equivariance_full_k_and_shift_invariance():
    rng = np.random.default_rng(2)
    z = rng.normal(size=(3, 50))
    perm = rng.permutation(50)
    idx, lp = orc.teacher_topk(z, 50)
    np.testing.assert_allclose(np.exp(lp).sum(axis=1), 1.0, atol=1e-13)     # k = V: the whole distribution
    idx_p, lp_p = orc.teacher_topk(z[:, perm], 5)
    idx5, lp5 = orc.teacher_topk(z, 5)
    assert (perm[idx_p] == idx5).all()                                      # no ties in a continuous draw
    np.testing.assert_allclose(lp_p, lp5, atol=1e-13)
    idx_s, lp_s = orc.teacher_topk(z + 11.0, 5)
    assert (idx_s == idx5).all()
    np.testing.assert_allclose(lp_s, lp5, atol=1e-12)


def test_records_feed_the_distillation_loss():
    """A student equal to the teacher: the truncated loss is 0 at full mass, and the rest-bucket
    loss is 0 for any k."""
    rng = np.random.default_rng(3)
    z = rng.normal(size=(4, 30)) * 2
    idx, lp = orc.teacher_topk(z, 30)
    assert abs(orc.distill_kl(z, idx, lp)[0]) < 1e-12
    idx, lp = orc.teacher_topk(z, 6)
    loss, g, _ = orc.distill_kl_rest_bucket(z, idx, lp)
    assert abs(loss) < 1e-12 and np.abs(g).max() < 1e-12
