"""CPU oracle for the learner-side scoring pass - TEST INFRASTRUCTURE, not a product path.

The policy update of the paper (Alg. 1, last step; the policy-gradient equation of Sec. 3) needs,
for every generated token y_t of a trajectory, log pi_theta(y_t | s_t, p, G): the log-probability of
that token under the full-vocabulary softmax of the decoder's logits at the preceding position.  The
objective sums A_{G,p}(tau) * log pi_theta(y_t) over the tokens player p produced, with the RAE
advantage A of that player and game and without normalising by response length; the
hyper-parameter table (App. D) adds a PPO-style policy clipping parameter 0.2 and two proximal
epochs, i.e. the clipped importance-ratio surrogate.  Written out:

    logp_t     = logits_{t-1}[y_t] - logsumexp_v(logits_{t-1}[v])
    reinforce  = sum_t mask_t * A_t * logp_t
    r_t        = exp(logp_t - logp_old_t)
    surrogate  = sum_t mask_t * min( r_t * A_t , clip(r_t, 1 - eps, 1 + eps) * A_t )

A_t is the advantage of the player who produced token t (the caller expands the per-trajectory,
per-role RAE advantages to tokens); mask_t selects generated tokens (prompt and observation tokens
carry no gradient).  Everything is float64.  Backward pass and optimiser are outside this build.
"""
from __future__ import annotations

import numpy as np

from . import decoder as od


def log_softmax_rows(logits: np.ndarray) -> np.ndarray:
    z = np.asarray(logits, dtype=np.float64)
    m = z.max(axis=-1, keepdims=True)
    return z - m - np.log(np.exp(z - m).sum(axis=-1, keepdims=True))


def token_logprobs(g, weights, tokens, dtype=np.float64) -> np.ndarray:
    """logp[i] = log pi(tokens[i+1] | tokens[0..i]), i = 0 .. T-2, by one full causal forward."""
    tokens = np.asarray(tokens, dtype=np.int64)
    T = tokens.shape[0]
    if T < 2:
        return np.zeros(0, dtype=np.float64)
    logits = od.forward_full(g, weights, tokens, logits_at=np.arange(T - 1), dtype=dtype)
    lsm = log_softmax_rows(logits)
    return lsm[np.arange(T - 1), tokens[1:]]


def reinforce_objective(logp: np.ndarray, adv: np.ndarray, mask: np.ndarray) -> float:
    return float(np.sum(np.asarray(mask, dtype=np.float64) * np.asarray(adv, dtype=np.float64) * np.asarray(logp, dtype=np.float64)))


def clipped_surrogate(logp_new: np.ndarray, logp_old: np.ndarray, adv: np.ndarray, mask: np.ndarray, eps: float = 0.2) -> float:
    ln = np.asarray(logp_new, dtype=np.float64)
    lo = np.asarray(logp_old, dtype=np.float64)
    A = np.asarray(adv, dtype=np.float64)
    r = np.exp(ln - lo)
    per_token = np.minimum(r * A, np.clip(r, 1.0 - eps, 1.0 + eps) * A)
    return float(np.sum(np.asarray(mask, dtype=np.float64) * per_token))
