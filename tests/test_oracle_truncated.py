"""Pins for the truncated-sampling oracle: hand-computed keep sets, reductions to the untruncated
sampler and to greedy, tie handling, and the sampled frequencies against the renormalised truncated
softmax."""
import numpy as np
import pytest

from oracle import sampling as osamp
from oracle import truncated as otr


def _logits_from_probs(p):
    return np.log(np.asarray(p, dtype=np.float64)).astype(np.float32)


def test_hand_computed_top_p_sets():
    lg = _logits_from_probs([0.05, 0.5, 0.15, 0.3])             # descending order: 1, 3, 2, 0
    assert otr.keep_mask(lg, 1.0, 0, 0.45).tolist() == [False, True, False, False]      # 0.5 >= 0.45
    assert otr.keep_mask(lg, 1.0, 0, 0.75).tolist() == [False, True, False, True]       # 0.5 < 0.75 <= 0.8
    assert otr.keep_mask(lg, 1.0, 0, 0.85).tolist() == [False, True, True, True]        # 0.8 < 0.85 <= 0.95
    assert otr.keep_mask(lg, 1.0, 0, 0.99).tolist() == [True, True, True, True]
    assert otr.keep_mask(lg, 1.0, 0, 1.0).all()


def test_hand_computed_top_k_then_top_p():
    lg = _logits_from_probs([0.05, 0.5, 0.15, 0.3])
    assert otr.keep_mask(lg, 1.0, 2, 1.0).tolist() == [False, True, False, True]
    # top-p sees the distribution renormalised over the two survivors: 0.625, 0.375
    assert otr.keep_mask(lg, 1.0, 2, 0.6).tolist() == [False, True, False, False]
    assert otr.keep_mask(lg, 1.0, 2, 0.7).tolist() == [False, True, False, True]
    # without top-k, 0.7 of the full distribution also needs the second token but 0.85 a third one
    assert otr.keep_mask(lg, 1.0, 3, 0.85).tolist() == [False, True, True, True]
    assert otr.keep_mask(lg, 1.0, 2, 0.85).tolist() == [False, True, False, True]


def test_temperature_sharpens_before_truncation():
    lg = _logits_from_probs([0.4, 0.35, 0.25])
    assert otr.keep_mask(lg, 1.0, 0, 0.7).tolist() == [True, True, False]       # 0.4 < 0.7 <= 0.75
    # T = 0.25: p ~ [0.568, 0.333, 0.087]... the first two still needed; T -> tiny: the first alone
    assert otr.keep_mask(lg, 0.02, 0, 0.7).tolist() == [True, False, False]


def test_ties_are_kept_or_dropped_together():
    lg = np.array([1.0, 3.0, 2.0, 2.0, 2.0, 0.0], dtype=np.float32)
    assert otr.keep_mask(lg, 1.0, 2, 1.0).tolist() == [False, True, True, True, True, False]   # the 2nd largest value is tied
    assert otr.keep_mask(lg, 1.0, 1, 1.0).tolist() == [False, True, False, False, False, False]
    p = otr.truncated_distribution(lg, 1.0, 0, 1.0)
    cut = float(p[1] + 0.5 * p[2])                                   # inside the tie group
    assert otr.keep_mask(lg, 1.0, 0, cut).tolist() == [False, True, True, True, True, False]


def test_untruncated_parameters_reduce_to_the_plain_sampler():
    rng = np.random.default_rng(0)
    for _ in range(20):
        V = int(rng.integers(2, 400))
        lg = rng.normal(size=V).astype(np.float32)
        g = osamp.gumbel_noise(3, 1, int(rng.integers(0, 100)), V)
        for T in (1.0, 0.6):
            want, wm = osamp.sample_row(lg, T, g)
            for k in (0, -1, V, V + 5):
                tok, m, tau, _ = otr.sample_row(lg, T, k, 1.0, g)
                assert tok == want and m == pytest.approx(wm) and tau == -np.inf


def test_top_k_one_is_greedy():
    rng = np.random.default_rng(1)
    for _ in range(20):
        V = int(rng.integers(2, 400))
        lg = rng.normal(size=V).astype(np.float32)
        g = osamp.gumbel_noise(4, 0, 0, V)
        tok, m, _, _ = otr.sample_row(lg, 0.8, 1, 1.0, g)
        assert tok == int(np.argmax(lg)) and m == np.inf


def test_keep_set_is_the_smallest_prefix_reaching_p():
    """Brute force on random rows: the keep set is a prefix of the descending order, its mass reaches p,
    and dropping its smallest score level would fall short."""
    rng = np.random.default_rng(2)
    for _ in range(50):
        V = int(rng.integers(3, 60))
        lg = (rng.normal(size=V) * 2).astype(np.float32)
        T = float(rng.choice([0.6, 1.0, 1.7]))
        p = float(rng.uniform(0.05, 0.999))
        k = int(rng.choice([0, 0, 5, V // 2 + 1]))
        z = otr.scaled(lg, T).astype(np.float64)
        base = np.ones(V, bool)
        if 0 < k < V:
            base = z >= np.sort(z)[::-1][k - 1]
        q = np.where(base, np.exp(z - z.max()), 0.0); q /= q.sum()
        m = otr.keep_mask(lg, T, k, p)
        _, slack = otr.keep_threshold(lg, T, k, p)
        assert m.any() and not (m & ~base).any()
        assert z[m].min() > z[~m & base].max() if (~m & base).any() else True          # a prefix of the order
        if slack < 1e-9:
            continue
        assert q[m].sum() >= p - 1e-12
        lowest = z[m].min()
        assert q[m & (z > lowest)].sum() < p + 1e-12


def test_sampled_frequencies_match_the_truncated_softmax():
    lg = np.array([2.0, 1.0, 0.5, 0.0, -1.0, -3.0], dtype=np.float32)
    T, k, p = 0.6, 5, 0.9
    want = otr.truncated_distribution(lg, T, k, p)
    assert want[-1] == 0.0 and 2 <= np.count_nonzero(want) <= 5
    N = 40000
    counts = np.zeros(len(lg))
    for step in range(N):
        g = osamp.gumbel_noise(7, 2, step, len(lg))
        counts[otr.sample_row(lg, T, k, p, g)[0]] += 1
    assert counts[want == 0].sum() == 0
    sel = want > 0
    chi2 = ((counts[sel] - N * want[sel]) ** 2 / (N * want[sel])).sum()
    assert chi2 < 25.0, (chi2, counts / N, want)         # dof <= 4: P(chi2 > 25) ~ 5e-5
