"""Pins for the scoring oracle: normalisation, the chain rule against the decoder oracle, an independent
library log-softmax, closed forms of the clipped surrogate, and a plain-loop brute force."""
import math

import numpy as np
import pytest
import scipy.special

from oracle import decoder as od
from oracle import scoring as osc
from paper_2506_24119_amd import inputs as si

G = si.ModelGeometry("score-tiny", 2, 64, 4, 2, 16, 128, 97, 1e4, qk_norm=True)


def test_log_softmax_matches_library_and_normalises():
    rng = np.random.default_rng(0)
    z = rng.normal(size=(5, 301)) * 7 + 100.0                 # large offset: the max subtraction matters
    got = osc.log_softmax_rows(z)
    assert np.allclose(got, scipy.special.log_softmax(z, axis=-1), rtol=0, atol=1e-12)
    assert np.allclose(np.exp(got).sum(axis=-1), 1.0, atol=1e-12)


def test_token_logprobs_chain_rule_and_shapes():
    w = si.make_weights(G, seed=3)
    toks = si.make_prompts(G.vocab, 1, 23, 23, seed=4)[0]
    lp = osc.token_logprobs(G, w, toks)
    assert lp.shape == (22,) and (lp < 0).all()
    # each entry from the definition: the decoder oracle's logits at the previous position
    for i in (0, 7, 21):
        lg = od.forward_full(G, w, toks[:i + 1], logits_at=[i])[0]
        want = lg[toks[i + 1]] - scipy.special.logsumexp(lg)
        assert lp[i] == pytest.approx(want, abs=1e-10)
    # a prefix of the sequence has the same conditionals (causality)
    assert np.allclose(osc.token_logprobs(G, w, toks[:10]), lp[:9], atol=1e-10)
    # probabilities of all possible next tokens sum to one
    total = 0.0
    for v in range(G.vocab):
        t2 = np.concatenate([toks[:5], [v]])
        total += math.exp(osc.token_logprobs(G, w, t2)[-1])
    assert total == pytest.approx(1.0, abs=1e-9)
    assert osc.token_logprobs(G, w, toks[:1]).shape == (0,)


def test_uniform_policy_closed_form():
    """All matrices zero except the embedding: logits are constant-free of context only through E;
    with a zero LM head every token has log-probability -ln V."""
    w = si.make_weights(G, seed=5)
    w = dict(w); w["lm_head"] = np.zeros_like(w["lm_head"])
    lp = osc.token_logprobs(G, w, np.arange(12) % G.vocab)
    assert np.allclose(lp, -math.log(G.vocab), atol=1e-12)


def test_surrogate_closed_forms():
    one = np.ones(1)
    A = 2.0
    for r, want in ((1.0, A), (1.1, 1.1 * A), (1.5, 1.2 * A), (0.5, 0.5 * A), (0.9, 0.9 * A)):      # A > 0: capped above
        assert osc.clipped_surrogate(np.log([r]), np.zeros(1), [A], one) == pytest.approx(want)
    for r, want in ((1.0, -A), (1.5, -1.5 * A), (0.5, -0.8 * A), (0.9, -0.9 * A), (1.1, -1.1 * A)):  # A < 0: floored below
        assert osc.clipped_surrogate(np.log([r]), np.zeros(1), [-A], one) == pytest.approx(want)
    # on-policy (ratio 1) the surrogate is the sum of advantages, and its value matches REINFORCE's weighting
    rng = np.random.default_rng(1)
    lp = -rng.uniform(0.1, 5, size=50); adv = rng.normal(size=50); mask = rng.integers(0, 2, size=50)
    assert osc.clipped_surrogate(lp, lp, adv, mask) == pytest.approx(float((mask * adv).sum()))
    assert osc.reinforce_objective(lp, adv, mask) == pytest.approx(float((mask * adv * lp).sum()))
    assert osc.clipped_surrogate(lp, lp, adv, np.zeros(50)) == 0.0
    # eps = 0 freezes the ratio at 1 wherever moving it would help
    assert osc.clipped_surrogate(np.log([1.3]), np.zeros(1), [1.0], one, eps=0.0) == pytest.approx(1.0)


def test_surrogate_brute_force():
    rng = np.random.default_rng(2)
    n = 200
    ln = -rng.uniform(0.05, 6, size=n); lo = ln + rng.normal(size=n) * 0.3
    adv = rng.normal(size=n); mask = rng.integers(0, 2, size=n)
    total = 0.0
    for i in range(n):
        if not mask[i]:
            continue
        r = math.exp(ln[i] - lo[i])
        rc = min(max(r, 0.8), 1.2)
        total += min(r * adv[i], rc * adv[i])
    assert osc.clipped_surrogate(ln, lo, adv, mask, 0.2) == pytest.approx(total, rel=1e-12)


def test_zero_sum_advantages_cancel_on_policy():
    """Two roles of one trajectory with RAE advantages A and -A (zero-sum game, Sec. 3): with equal token
    counts the on-policy surrogate is zero."""
    adv = np.array([0.7] * 6 + [-0.7] * 6)
    lp = -np.linspace(0.1, 3, 12)
    assert osc.clipped_surrogate(lp, lp, adv, np.ones(12)) == pytest.approx(0.0, abs=1e-12)
