"""Pins for oracle/rae.py: the paper's recurrence against closed forms, the
zero-sum symmetry, limiting cases and a hand-computed worked example."""
import os

import numpy as np

from oracle.rae import RAE
from paper_2506_24119_amd import inputs as si

GOLD = os.path.join(os.path.dirname(__file__), "golden", "rae_alpha095_worked.txt")


def test_worked_example_alpha_095():
    rows = np.loadtxt(GOLD)
    r = RAE(1, 0.95)
    for R0, b0, a0, b1, a1 in rows:
        adv = r.update([0], [R0])
        np.testing.assert_allclose(r.b[0], [b0, b1], rtol=0, atol=1e-15)
        np.testing.assert_allclose(adv[0], [a0, a1], rtol=0, atol=1e-15)


def test_constant_reward_closed_form():
    # b_n = R (1 - alpha^n), A_n = R alpha^n   (geometric series of the EMA from b_0 = 0)
    alpha, R, n = 0.95, 1.0, 40
    r = RAE(2, alpha)
    adv = r.update(np.ones(n, dtype=np.int32), np.full(n, R))
    k = np.arange(1, n + 1)
    np.testing.assert_allclose(adv[:, 0], R * alpha ** k, rtol=1e-12)
    np.testing.assert_allclose(adv[:, 1], -R * alpha ** k, rtol=1e-12)
    np.testing.assert_allclose(r.b[1], [R * (1 - alpha ** n), -R * (1 - alpha ** n)], rtol=1e-12)
    assert np.array_equal(r.b[0], [0.0, 0.0])              # the other game never moved


def test_general_closed_form_and_order_dependence():
    gid, R0 = si.make_game_outcomes(1, 50, seed=1)
    alpha = 0.9
    r = RAE(1, alpha)
    adv = r.update(gid, R0)
    n = len(R0)
    for i in (0, 7, n - 1):
        b = (1 - alpha) * sum(alpha ** (i - k) * R0[k] for k in range(i + 1))
        assert abs(adv[i, 0] - (R0[i] - b)) < 1e-13
    # the advantage uses the baseline AFTER its own update: first A is R - (1-alpha) R = alpha R
    first = int(np.flatnonzero(R0)[0])
    r2 = RAE(1, alpha)
    a2 = r2.update([0], [R0[first]])
    assert abs(a2[0, 0] - alpha * R0[first]) < 1e-15


def test_zero_sum_symmetry_and_game_independence():
    gid, R0 = si.make_game_outcomes(3, 200, seed=2)
    r = RAE(3, 0.95)
    adv = r.update(gid, R0)
    np.testing.assert_allclose(adv[:, 1], -adv[:, 0], atol=1e-15)
    np.testing.assert_allclose(r.b[:, 1], -r.b[:, 0], atol=1e-15)
    # games never interact: running each game's subsequence alone gives the same numbers
    for G in range(3):
        sel = gid == G
        solo = RAE(1, 0.95)
        a = solo.update(np.zeros(sel.sum(), dtype=np.int32), R0[sel])
        np.testing.assert_allclose(a, adv[sel], atol=1e-15)
        np.testing.assert_allclose(solo.b[0], r.b[G], atol=1e-15)


def test_limits_alpha_zero_and_one():
    gid, R0 = si.make_game_outcomes(2, 30, seed=3)
    assert np.array_equal(RAE(2, 0.0).update(gid, R0), np.zeros((30, 2)))      # baseline = last reward
    a1 = RAE(2, 1.0).update(gid, R0)                                            # baseline frozen at 0
    assert np.array_equal(a1[:, 0], R0) and np.array_equal(a1[:, 1], -R0)


def test_split_batches_equal_one_batch():
    gid, R0 = si.make_game_outcomes(3, 64, seed=4)
    a = RAE(3).update(gid, R0)
    r = RAE(3)
    b = np.concatenate([r.update(gid[:10], R0[:10]), r.update(gid[10:], R0[10:])])
    assert np.array_equal(a, b)
