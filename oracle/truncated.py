"""CPU oracle for truncated (top-k / top-p) temperature sampling - TEST INFRASTRUCTURE, not a product path.

The evaluation runs of the paper decode with temperature 0.6 and top-p 0.95 (appendix
"Evaluation Settings"); the actor's top-p = 1.0, top-k = -1 (appendix "Hyperparameter
Configuration") is the untruncated special case.  The paper gives the parameters, not an algorithm;
the definition below is the usual one, with every choice it leaves open stated:

    z_v = fp32(logit_v) / fp32(T)                                   (T > 0)
    top-k (0 < k < V):  tau_k = the k-th largest z (with multiplicity); keep z_v >= tau_k
    top-p (p < 1):      over the tokens top-k kept, q_v = exp(z_v - max z) / Z;  walk them in
                        descending order of z and stop at the first token where the running sum of q
                        reaches p;  tau_p = that token's z;  keep z_v >= tau_p
    keep set           = { v : z_v >= max(tau_k, tau_p) }    - equal scores are kept or dropped together,
                        so the set does not depend on how ties are ordered
    token              = argmax over the keep set of z_v + g_v, g standard Gumbel, lowest index on ties

top-k is applied before top-p and top-p sees the distribution renormalised over the top-k survivors.
Drawing the argmax of z + g over a subset is an exact draw from softmax(z) renormalised over that
subset, so this samples the truncated categorical exactly.  Running sums are float64 here; `slack`
tells a caller how close the running sum came to p on either side of the cut (relative to Z), so that
a comparison against an implementation that adds in another order can skip the undecidable cases.
"""
from __future__ import annotations

import numpy as np


def scaled(logits_row: np.ndarray, temperature: float) -> np.ndarray:
    assert temperature > 0.0
    return np.asarray(logits_row).astype(np.float32) / np.float32(temperature)


def keep_threshold(logits_row: np.ndarray, temperature: float, top_k: int, top_p: float):
    """(tau, slack): the keep set is scaled(logits) >= tau; tau = -inf when nothing is cut."""
    z = scaled(logits_row, temperature)
    V = z.shape[0]
    zs = np.sort(z)[::-1]                       # descending
    tau = np.float32(-np.inf)
    n = V
    if 0 < top_k < V:
        tau = zs[top_k - 1]
        n = int(np.count_nonzero(z >= tau))     # ties of the k-th value stay in
    slack = np.inf
    if top_p < 1.0:
        kept = zs[:n].astype(np.float64)
        w = np.exp(kept - kept[0])
        c = np.cumsum(w)
        target = float(top_p) * c[-1]
        idx = int(np.searchsorted(c, target, side="left"))      # first index with c[idx] >= target
        idx = min(idx, n - 1)
        tau_p = zs[idx]
        below = c[idx - 1] if idx > 0 else 0.0
        slack = min(abs(c[idx] - target), abs(target - below)) / c[-1]
        tau = max(tau, tau_p)
    return np.float32(tau), float(slack)


def keep_mask(logits_row: np.ndarray, temperature: float, top_k: int, top_p: float) -> np.ndarray:
    tau, _ = keep_threshold(logits_row, temperature, top_k, top_p)
    return scaled(logits_row, temperature) >= tau


def truncated_distribution(logits_row: np.ndarray, temperature: float, top_k: int, top_p: float) -> np.ndarray:
    """Probabilities (float64) of the truncated, renormalised categorical."""
    z = scaled(logits_row, temperature).astype(np.float64)
    m = keep_mask(logits_row, temperature, top_k, top_p)
    w = np.where(m, np.exp(z - z[m].max()), 0.0)
    return w / w.sum()


def sample_row(logits_row: np.ndarray, temperature: float, top_k: int, top_p: float, noise_row: np.ndarray):
    """(token, margin, tau, slack).  margin = gap between the two largest perturbed scores inside the
    keep set (inf when one token is kept)."""
    z = scaled(logits_row, temperature)
    tau, slack = keep_threshold(logits_row, temperature, top_k, top_p)
    s = z + np.asarray(noise_row, dtype=np.float32)
    s = np.where(z >= tau, s, np.float32(-np.inf))
    tok = int(np.argmax(s))
    kept = s[z >= tau]
    margin = np.inf if kept.shape[0] < 2 else float(np.diff(np.partition(kept, -2)[-2:])[0])
    return tok, margin, tau, slack
