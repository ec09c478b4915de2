"""CPU oracle for the policy decoder — TEST INFRASTRUCTURE, not a product path.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It shares no code with the HIP path and never imports it.

What it computes: the paper generates every turn's response by sampling
y ~ pi_theta(. | s) token by token (Sec. 3, "Self-play"; Alg. 1, the generation
step), with the actor settings of the hyper-parameter table in App. D
(temperature 1.0, top-p 1.0, top-k -1: an untruncated categorical).  The paper
does not spell out the transformer; the decoder below is the textbook
pre-norm GQA/RoPE/SwiGLU decoder of the model families it names (Sec. 4,
"Models"), written as the plain definition:

    logits at position t  =  one full causal forward over tokens 0..t.

`forward_full` is that definition (explicit T x T masked softmax, no cache, no
blocking).  `CachedDecoder` is the straightforward KV-cached loop; the tests
pin it to `forward_full`, and pin `forward_full` to closed forms, special
cases and an independent library implementation.

All arithmetic is float64 by default (`dtype=np.float32` gives the fp32
variant).  Weights are taken exactly as given: fp32 arrays, or bf16 bit
patterns (uint16) widened exactly.

Parity pins: every function here is pinned by tests/test_oracle_*.py except
the numerical values of full-size logits, which nothing in the paper fixes
("parity unpinned" beyond the oracle's own pins on small shapes).
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np


# ----------------------------------------------------------------------------
# storage format
# ----------------------------------------------------------------------------
def widen(w: np.ndarray, dtype=np.float64) -> np.ndarray:
    """Weights as `dtype` values: uint16 arrays are bf16 bit patterns (upper
    half of an IEEE fp32), anything else is numeric already."""
    if w.dtype == np.uint16:
        return (w.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(dtype)
    return w.astype(dtype, copy=False)


# ----------------------------------------------------------------------------
# building blocks (each over the last axis / in the paper-family's convention)
# ----------------------------------------------------------------------------
def rmsnorm(v: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """v / sqrt(mean(v^2) + eps) * gain over the last axis."""
    ms = np.mean(v * v, axis=-1, keepdims=True)
    return v / np.sqrt(ms + eps) * gain


def rope(x: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, "rotate-half" pairing.  x: [T, H, hd]; positions: [T].
    Pair (j, j + hd/2) is rotated by the angle pos * theta^(-2j/hd)."""
    hd = x.shape[-1]
    half = hd // 2
    j = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * j / hd)
    ang = positions.astype(np.float64)[:, None] * inv_freq[None, :]          # [T, half]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def causal_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """q: [T, Hq, hd], k/v: [T, Hkv, hd].  Query head h reads kv head h // G.
    Explicit T x T scores, lower-triangular mask, max-subtracted softmax."""
    T, hq, hd = q.shape
    hkv = k.shape[1]
    G = hq // hkv
    out = np.empty_like(q)
    mask = np.tril(np.ones((T, T), dtype=bool))
    for h in range(hq):
        kv = h // G
        s = (q[:, h, :] @ k[:, kv, :].T) / np.sqrt(np.asarray(hd, dtype=q.dtype))
        s = np.where(mask, s, -np.inf)
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=-1, keepdims=True)
        out[:, h, :] = p @ v[:, kv, :]
    return out


def single_query_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """One new position against a cache.  q: [Hq, hd]; k/v: [n, Hkv, hd]
    (all n cached positions are visible)."""
    hq, hd = q.shape
    G = hq // k.shape[1]
    out = np.empty_like(q)
    for h in range(hq):
        kv = h // G
        s = (k[:, kv, :] @ q[h]) / np.sqrt(np.asarray(hd, dtype=q.dtype))
        s = s - s.max()
        p = np.exp(s)
        p = p / p.sum()
        out[h] = p @ v[:, kv, :]
    return out


# ----------------------------------------------------------------------------
# the model
# ----------------------------------------------------------------------------
class _Layer:
    def __init__(self, lw: Dict[str, np.ndarray], dtype):
        for name, arr in lw.items():
            setattr(self, name, widen(arr, dtype))
        for opt in ("bq", "bk", "bv", "q_norm", "k_norm"):
            if not hasattr(self, opt):
                setattr(self, opt, None)


def _qkv(g, L: _Layer, h: np.ndarray, positions: np.ndarray):
    """Projections, optional bias, optional per-head RMSNorm (before RoPE), RoPE."""
    T = h.shape[0]
    q = h @ L.wq.T
    k = h @ L.wk.T
    v = h @ L.wv.T
    if L.bq is not None:
        q, k, v = q + L.bq, k + L.bk, v + L.bv
    q = q.reshape(T, g.n_q_heads, g.head_dim)
    k = k.reshape(T, g.n_kv_heads, g.head_dim)
    v = v.reshape(T, g.n_kv_heads, g.head_dim)
    if L.q_norm is not None:
        q = rmsnorm(q, L.q_norm, g.rms_eps)
        k = rmsnorm(k, L.k_norm, g.rms_eps)
    q = rope(q, positions, g.rope_theta)
    k = rope(k, positions, g.rope_theta)
    return q, k, v


def _mlp(L: _Layer, h: np.ndarray) -> np.ndarray:
    return (silu(h @ L.w_gate.T) * (h @ L.w_up.T)) @ L.w_down.T


def forward_full(g, weights: Dict[str, object], tokens: Sequence[int],
                 logits_at: Optional[Sequence[int]] = None, dtype=np.float64) -> np.ndarray:
    """Logits of one sequence by a full causal forward: the plain definition.

    Returns [len(logits_at), vocab] (default: every position).  Row i holds the
    next-token logits after consuming tokens[0 .. logits_at[i]]."""
    tokens = np.asarray(tokens, dtype=np.int64)
    T = tokens.shape[0]
    pos = np.arange(T)
    x = widen(weights["embed"][tokens], dtype)
    for lw in weights["layers"]:
        L = _Layer(lw, dtype)
        h = rmsnorm(x, L.attn_norm, g.rms_eps)
        q, k, v = _qkv(g, L, h, pos)
        o = causal_attention(q, k, v).reshape(T, g.n_q_heads * g.head_dim)
        x = x + o @ L.wo.T
        x = x + _mlp(L, rmsnorm(x, L.mlp_norm, g.rms_eps))
    sel = np.arange(T) if logits_at is None else np.asarray(logits_at, dtype=np.int64)
    hf = rmsnorm(x[sel], widen(weights["final_norm"], dtype), g.rms_eps)
    return hf @ widen(weights["lm_head"], dtype).T


def forward_full_many(g, weights: Dict[str, object], sequences: Sequence[Sequence[int]],
                      logits_at: Sequence[Sequence[int]], dtype=np.float64, progress=None) -> List[np.ndarray]:
    """forward_full for several independent sequences, visiting each layer once so that its weights
    are widened once (the only difference from calling forward_full per sequence)."""
    toks = [np.asarray(t, dtype=np.int64) for t in sequences]
    xs = [widen(weights["embed"][t], dtype) for t in toks]
    for li, lw in enumerate(weights["layers"]):
        L = _Layer(lw, dtype)
        for i, t in enumerate(toks):
            T = t.shape[0]
            x = xs[i]
            h = rmsnorm(x, L.attn_norm, g.rms_eps)
            q, k, v = _qkv(g, L, h, np.arange(T))
            o = causal_attention(q, k, v).reshape(T, g.n_q_heads * g.head_dim)
            x = x + o @ L.wo.T
            xs[i] = x + _mlp(L, rmsnorm(x, L.mlp_norm, g.rms_eps))
        if progress is not None:
            progress(li)
    fn = widen(weights["final_norm"], dtype)
    lm = widen(weights["lm_head"], dtype)
    return [rmsnorm(xs[i][np.asarray(logits_at[i], dtype=np.int64)], fn, g.rms_eps) @ lm.T for i in range(len(toks))]


class CachedDecoder:
    """KV-cached incremental decoding of ONE sequence (contiguous cache).

    prefill(tokens) consumes a prompt and returns the logits after its last
    token; step(token) consumes one more token.  Convention: the k-th decode
    step consumes the k-th generated token at position len(prompt) + k."""

    def __init__(self, g, weights: Dict[str, object], dtype=np.float64):
        self.g = g
        self.dtype = dtype
        self.w = weights
        self.layers = [_Layer(lw, dtype) for lw in weights["layers"]]
        self.final_norm = widen(weights["final_norm"], dtype)
        self.lm_head = widen(weights["lm_head"], dtype)
        self.k: List[np.ndarray] = [np.zeros((0, g.n_kv_heads, g.head_dim), dtype) for _ in self.layers]
        self.v: List[np.ndarray] = [np.zeros((0, g.n_kv_heads, g.head_dim), dtype) for _ in self.layers]
        self.n = 0

    def _advance(self, tokens: np.ndarray) -> np.ndarray:
        g = self.g
        T = tokens.shape[0]
        pos = np.arange(self.n, self.n + T)
        x = widen(self.w["embed"][tokens], self.dtype)
        for i, L in enumerate(self.layers):
            h = rmsnorm(x, L.attn_norm, g.rms_eps)
            q, k, v = _qkv(g, L, h, pos)
            self.k[i] = np.concatenate([self.k[i], k], axis=0)
            self.v[i] = np.concatenate([self.v[i], v], axis=0)
            o = np.empty_like(q)
            for t in range(T):               # position self.n + t sees the cache up to itself
                n_vis = self.n + t + 1
                o[t] = single_query_attention(q[t], self.k[i][:n_vis], self.v[i][:n_vis])
            x = x + o.reshape(T, -1) @ L.wo.T
            x = x + _mlp(L, rmsnorm(x, L.mlp_norm, g.rms_eps))
        self.n += T
        return rmsnorm(x[-1], self.final_norm, g.rms_eps) @ self.lm_head.T

    def prefill(self, tokens: Sequence[int]) -> np.ndarray:
        return self._advance(np.asarray(tokens, dtype=np.int64))

    def step(self, token: int) -> np.ndarray:
        return self._advance(np.asarray([token], dtype=np.int64))
