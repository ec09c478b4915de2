"""CPU oracle for seeded temperature sampling — TEST INFRASTRUCTURE, not a product path.

The actor samples from the untruncated categorical softmax(logits / T) with
T = 1.0, top-p = 1.0, top-k = -1 (hyper-parameter table, App. D, "Actor").
Drawing argmax_v(logits_v / T + g_v) with i.i.d. standard Gumbel g_v is that
same distribution (Gumbel-max), and greedy decoding is the g = 0 case.

The noise stream is this build's own specification (the paper fixes the
distribution, not a generator): a stateless counter-based generator keyed by
(seed, seq_id, step, v) so that any element can be produced independently.

    mix(z):  z ^= z >> 30;  z *= 0xBF58476D1CE4E5B9
             z ^= z >> 27;  z *= 0x94D049BB133111EB
             z ^= z >> 31                              (all mod 2^64)
    key  = mix( mix(seed ^ 0x9E3779B97F4A7C15) + (seq_id << 32 | step) )
    r    = mix( key + v * 0x9E3779B97F4A7C15 ) >> 32            (32 bits)
    u    = ((r >> 9) + 0.5) * 2^-23                             in (0, 1)
    g    = -ln(-ln(u))                                          in fp32

The decision (argmax) is taken in fp32, the precision the kernel uses: scores
are fp32(logits) / fp32(T) + g, ties go to the lowest index.
"""
from __future__ import annotations

import numpy as np

_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_GOLD = np.uint64(0x9E3779B97F4A7C15)


def _mix(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def random_bits(seed: int, seq_id: int, step: int, vocab: int) -> np.ndarray:
    """The 32-bit outputs r[v], v in [0, vocab), for one (seed, seq_id, step)."""
    with np.errstate(over="ignore"):
        key = _mix(_mix(np.uint64(seed) ^ _GOLD)
                   + ((np.uint64(seq_id) << np.uint64(32)) | np.uint64(step)))
        v = np.arange(vocab, dtype=np.uint64)
        r = _mix(key + v * _GOLD) >> np.uint64(32)
    return r.astype(np.uint32)


def uniform_from_bits(r: np.ndarray) -> np.ndarray:
    """Top 23 bits -> the open interval (0, 1).  Every value k + 0.5, k < 2^23,
    fits fp32's 24-bit significand exactly, so u is never rounded to 0 or 1
    (with 24 bits the largest value would round up to 1 and give infinite noise)."""
    return ((r >> np.uint32(9)).astype(np.float32) + np.float32(0.5)) * np.float32(2.0 ** -23)


def gumbel_noise(seed: int, seq_id: int, step: int, vocab: int) -> np.ndarray:
    """Standard Gumbel noise g[v] in fp32 for one row."""
    u = uniform_from_bits(random_bits(seed, seq_id, step, vocab))
    return (-np.log(-np.log(u, dtype=np.float32), dtype=np.float32)).astype(np.float32)


def scores(logits_row: np.ndarray, temperature: float, noise_row) -> np.ndarray:
    """fp32 perturbed scores logits / T + g (greedy: the fp32 logits themselves)."""
    s = np.asarray(logits_row).astype(np.float32)
    if temperature > 0.0:
        s = s / np.float32(temperature) + np.asarray(noise_row, dtype=np.float32)
    return s


def sample_row(logits_row: np.ndarray, temperature: float, noise_row=None):
    """(token, margin): argmax of the scores (lowest index on ties) and the gap
    between the largest and second-largest score."""
    s = scores(logits_row, temperature, noise_row)
    tok = int(np.argmax(s))
    if s.shape[0] == 1:
        return tok, np.inf
    top2 = np.partition(s, -2)[-2:]
    return tok, float(top2[1] - top2[0])


def sample(logits: np.ndarray, temperature: float, seed: int, seq_ids, steps, noise=None):
    """Rows of `logits` [B, V] -> (tokens[B], margins[B]).  `noise` [B, V], when
    given, replaces the generated stream (the shared-noise test mode)."""
    B, V = logits.shape
    toks = np.empty(B, dtype=np.int32)
    margins = np.empty(B, dtype=np.float64)
    for b in range(B):
        g = None
        if temperature > 0.0:
            g = noise[b] if noise is not None else gumbel_noise(seed, int(seq_ids[b]), int(steps[b]), V)
        toks[b], margins[b] = sample_row(logits[b], temperature, g)
    return toks, margins
