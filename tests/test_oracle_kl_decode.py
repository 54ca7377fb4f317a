"""Pins for the distillation-loss oracle and the decode oracle.  CPU only."""
import json
import math
import os

import numpy as np
import pytest
from scipy import special

from oracle import cartridge_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------------------------------------
# loss
# ---------------------------------------------------------------------------------------------
def test_kl_hand_worked_example():
    with open(os.path.join(GOLDEN, "kl_worked_example.json")) as f:
        g = json.load(f)
    logits = np.log(np.array(g["logits_ln_of"]))[None, :]
    idx = np.array([g["teacher_idx"]])
    logp = np.log(np.array([g["teacher_prob"]]))
    loss, dl, row = orc.distill_kl(logits, idx, logp, scale=1.0)
    expect = sum(c * math.log(r) for c, r in g["kl_terms_ln_of"])
    assert abs(loss - expect) < 1e-14
    assert abs(row[0] - expect) < 1e-14
    np.testing.assert_allclose(dl[0], g["d_logits"], rtol=1e-13, atol=1e-15)


def test_full_teacher_is_textbook_kl():
    """k = |V| with the whole teacher distribution: Eq. 3's KL(teacher || student), computed here
    with scipy's rel_entr / log_softmax."""
    rng = np.random.default_rng(1)
    N, V = 6, 13
    z = rng.normal(0, 2, (N, V))
    t_logits = rng.normal(0, 2, (N, V))
    t = special.softmax(t_logits, axis=1)
    idx = np.stack([rng.permutation(V) for _ in range(N)])
    logp = np.log(np.take_along_axis(t, idx, axis=1))
    loss, dl, row = orc.distill_kl(z, idx, logp, scale=1.0)
    s = special.softmax(z, axis=1)
    ref_rows = special.rel_entr(t, s).sum(axis=1)
    np.testing.assert_allclose(row, ref_rows, rtol=1e-12)
    assert abs(loss - ref_rows.sum()) < 1e-12
    np.testing.assert_allclose(dl, s - t, rtol=1e-11, atol=1e-14)


def test_k1_is_cross_entropy():
    """One teacher entry with probability 1 is the next-token-prediction ablation of App. A.2:
    loss = -log s_y, gradient = s - onehot(y)."""
    rng = np.random.default_rng(2)
    N, V = 5, 9
    z = rng.normal(0, 3, (N, V))
    y = rng.integers(0, V, (N, 1))
    loss, dl, row = orc.distill_kl(z, y, np.zeros((N, 1)), scale=1.0 / N)
    ls = special.log_softmax(z, axis=1)
    ce = -np.take_along_axis(ls, y, axis=1)[:, 0]
    np.testing.assert_allclose(row, ce, rtol=1e-12)
    assert abs(loss - ce.mean()) < 1e-12
    onehot = np.zeros((N, V))
    onehot[np.arange(N), y[:, 0]] = 1.0
    np.testing.assert_allclose(dl, (np.exp(ls) - onehot) / N, rtol=1e-11, atol=1e-15)


def _teacher(rng, N, V, k, mass):
    idx = np.stack([rng.choice(V, k, replace=False) for _ in range(N)])
    w = special.softmax(rng.normal(0, 2, (N, k)), axis=1) * mass
    return idx, np.log(w)


def test_gradient_rows_sum_to_zero_and_shift_invariance():
    rng = np.random.default_rng(3)
    N, V, k = 7, 40, 6
    z = rng.normal(0, 2, (N, V))
    idx, logp = _teacher(rng, N, V, k, 0.9)
    loss, dl, row = orc.distill_kl(z, idx, logp, scale=0.3)
    assert np.abs(dl.sum(axis=1)).max() < 1e-15 * V * 10
    loss2, dl2, row2 = orc.distill_kl(z + rng.normal(size=(N, 1)) * 5, idx, logp, scale=0.3)
    assert abs(loss - loss2) < 1e-12
    np.testing.assert_allclose(dl, dl2, rtol=1e-10, atol=1e-14)


def test_lower_bound_and_its_minimiser():
    """With recorded mass M < 1 the truncated objective is >= M log M, attained when the student
    puts t/M on the recorded tokens; its gradient vanishes there."""
    rng = np.random.default_rng(4)
    N, V, k, M = 4, 12, 5, 0.9
    idx, logp = _teacher(rng, N, V, k, M)
    z = rng.normal(0, 2, (N, V))
    _, _, row = orc.distill_kl(z, idx, logp)
    assert (row >= M * math.log(M) - 1e-12).all()
    z_star = np.full((N, V), -np.inf)
    np.put_along_axis(z_star, idx, logp - math.log(M) + 3.0, axis=1)
    with np.errstate(invalid="ignore"):
        loss, dl, row = orc.distill_kl(z_star, idx, logp)
    np.testing.assert_allclose(row, M * math.log(M), rtol=1e-12)
    assert np.abs(np.nan_to_num(dl)).max() < 1e-15


def test_student_equal_to_teacher_gives_zero_loss_and_gradient():
    """Mass-1 teacher, student equal to it on the support and zero elsewhere: KL = 0, g = 0."""
    rng = np.random.default_rng(5)
    N, V, k = 3, 15, 4
    idx, logp = _teacher(rng, N, V, k, 1.0)
    z = np.full((N, V), -np.inf)
    np.put_along_axis(z, idx, logp + 2.5, axis=1)
    loss, dl, row = orc.distill_kl(z, idx, logp)
    assert abs(loss) < 1e-14
    assert np.abs(dl).max() < 1e-15
    # with M < 1 the value at s = t on the support is still exactly 0
    idx, logp = _teacher(rng, N, V, k, 0.8)
    zz = np.full((N, V), -30.0)
    np.put_along_axis(zz, idx, logp, axis=1)
    rest = (V - k)
    zz[zz == -30.0] = math.log(0.2 / rest)
    _, _, row = orc.distill_kl(zz, idx, logp)
    assert np.abs(row).max() < 1e-13


def test_kl_finite_differences_and_ignored_entries():
    rng = np.random.default_rng(6)
    N, V, k = 3, 11, 4
    z = rng.normal(0, 2, (N, V))
    idx, logp = _teacher(rng, N, V, k, 0.9)
    idx[1, 2] = -1                                    # ignored entry
    loss, dl, _ = orc.distill_kl(z, idx, logp, scale=0.5)
    eps = 1e-6
    num = np.zeros_like(z)
    for n in range(N):
        for v in range(V):
            zp = z.copy(); zp[n, v] += eps
            zm = z.copy(); zm[n, v] -= eps
            num[n, v] = (orc.distill_kl(zp, idx, logp, 0.5)[0] - orc.distill_kl(zm, idx, logp, 0.5)[0]) / (2 * eps)
    assert np.abs(num - dl).max() < 1e-8
    # the ignored entry contributes nothing: dropping its column gives the same numbers
    keep = [0, 1, 3]
    only = orc.distill_kl(z[1:2], idx[1:2, keep], logp[1:2, keep], 0.5)
    full_row = orc.distill_kl(z[1:2], idx[1:2], logp[1:2], 0.5)
    assert abs(only[0] - full_row[0]) < 1e-15
    np.testing.assert_allclose(only[1][0], dl[1], rtol=1e-13, atol=1e-16)


# ---------------------------------------------------------------------------------------------
# decode
# ---------------------------------------------------------------------------------------------
def _decode_problem(rng, B, Hq, Hkv, d, p, lens):
    cu = np.concatenate([[0], np.cumsum(lens)])
    T = int(cu[-1])
    return dict(q=rng.normal(size=(B, Hq, d)), z_k=rng.normal(size=(Hkv, p, d)),
                z_v=rng.normal(size=(Hkv, p, d)), k_own=rng.normal(size=(T, Hkv, d)),
                v_own=rng.normal(size=(T, Hkv, d)), cu_lens=cu)


def test_decode_is_last_row_of_training_attention():
    rng = np.random.default_rng(30)
    B, Hq, Hkv, d, p = 3, 4, 2, 5, 6
    lens = [4, 1, 7]
    pr = _decode_problem(rng, B, Hq, Hkv, d, p, lens)
    o, lse = orc.decode(**pr)
    for b, n in enumerate(lens):
        lo, hi = pr["cu_lens"][b], pr["cu_lens"][b + 1]
        qq = rng.normal(size=(1, n, Hq, d))
        qq[0, -1] = pr["q"][b]
        of, lf = orc.attn_fwd(qq, pr["k_own"][None, lo:hi], pr["v_own"][None, lo:hi], pr["z_k"], pr["z_v"])
        np.testing.assert_allclose(o[b], of[0, -1], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(lse[b], lf[0, :, -1], rtol=1e-12, atol=1e-14)


def test_decode_p0_is_plain_single_query_attention():
    rng = np.random.default_rng(31)
    pr = _decode_problem(rng, 2, 2, 2, 3, 0, [5, 2])
    o, lse = orc.decode(**pr, scale=0.4)
    for b in range(2):
        lo, hi = pr["cu_lens"][b], pr["cu_lens"][b + 1]
        for h in range(2):
            ws = [math.exp(0.4 * float(pr["q"][b, h] @ pr["k_own"][t, h])) for t in range(lo, hi)]
            ref = sum(w * pr["v_own"][t, h] for w, t in zip(ws, range(lo, hi))) / sum(ws)
            np.testing.assert_allclose(o[b, h], ref, rtol=1e-12)
            assert abs(lse[b, h] - math.log(sum(ws))) < 1e-12


def test_decode_lse_merge_identity():
    """Attention over [prefix ; own] == the LSE-weighted merge of attention over each part."""
    rng = np.random.default_rng(32)
    B, Hq, Hkv, d, p = 2, 4, 1, 4, 5
    pr = _decode_problem(rng, B, Hq, Hkv, d, p, [3, 6])
    o, lse = orc.decode(**pr)
    empty = np.zeros((Hkv, 0, d))
    o_own, l_own = orc.decode(pr["q"], empty, empty, pr["k_own"], pr["v_own"], pr["cu_lens"])
    # prefix alone: give every request one own token and remove its effect analytically is
    # awkward; instead use the training oracle with the prefix as the "own" keys of length p
    # and read the last row of a non-causal-equivalent: all p keys visible to row p-1.
    for b in range(B):
        qq = np.zeros((1, p, Hq, d)); qq[0, -1] = pr["q"][b]
        o_pre, l_pre = orc.attn_fwd(qq, pr["z_k"].transpose(1, 0, 2)[None], pr["z_v"].transpose(1, 0, 2)[None],
                                    empty, empty)
        o_pre, l_pre = o_pre[0, -1], l_pre[0, :, -1]
        m = np.maximum(l_pre, l_own[b])
        w1, w2 = np.exp(l_pre - m), np.exp(l_own[b] - m)
        merged = (w1[:, None] * o_pre + w2[:, None] * o_own[b]) / (w1 + w2)[:, None]
        np.testing.assert_allclose(o[b], merged, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(lse[b], m + np.log(w1 + w2), rtol=1e-12)
