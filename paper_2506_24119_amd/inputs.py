"""Seeded synthetic inputs for the self-play decode path.

This module only *draws data*: model geometries, random-init weights, prompt
token ids, ragged prompt lengths, physical page orders and zero-sum game
outcomes.  It holds none of the decoder's or the sampler's arithmetic, and it
is the only module that both the CPU oracle's tests and the HIP path's tests
use.  Everything is reproducible from the stated seeds.

The shapes stand in for the paper's self-play workload (Sec. 4 and the
hyper-parameter table of App. D): 128 samples per step, temperature 1.0,
untruncated sampling, prompts that are concatenated multi-turn game histories.
Token ids are uniform random and weights are random-init because neither the
game environments, the tokenizer nor the trained checkpoints are available.
"""
from __future__ import annotations

from dataclasses import dataclass, field, asdict
from typing import Dict, List, Optional, Tuple

import numpy as np

WEIGHT_FP32 = 0
WEIGHT_BF16 = 1


@dataclass(frozen=True)
class ModelGeometry:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int
    vocab: int
    rope_theta: float
    rms_eps: float = 1e-6
    qk_norm: bool = False
    qkv_bias: bool = False
    tie_lm_head: bool = True
    weight_dtype: int = WEIGHT_BF16
    kv_block_tokens: int = 16

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def params_per_layer(self) -> int:
        d, hq, hkv, hd, f = self.d_model, self.n_q_heads, self.n_kv_heads, self.head_dim, self.ffn_dim
        return d * (hq + 2 * hkv) * hd + hq * hd * d + 3 * d * f


@dataclass(frozen=True)
class Workload:
    """One of the benchmark configurations: a geometry plus a batch recipe."""
    key: str
    geometry: ModelGeometry
    batch: int
    prompt_lo: int
    prompt_hi: int          # inclusive
    decode_steps: int
    temperature: float      # 0 => greedy
    seed: int


GEOMETRIES: Dict[str, ModelGeometry] = {
    "tiny": ModelGeometry("tiny", 2, 128, 4, 2, 32, 512, 1024, 1e4,
                          weight_dtype=WEIGHT_FP32),
    "qwen3-0.6b": ModelGeometry("qwen3-0.6b", 28, 1024, 16, 8, 128, 3072, 151936, 1e6,
                                qk_norm=True),
    "qwen3-4b": ModelGeometry("qwen3-4b", 36, 2560, 32, 8, 128, 9728, 151936, 1e6,
                              qk_norm=True),
    "qwen2.5-7b": ModelGeometry("qwen2.5-7b", 28, 3584, 28, 4, 128, 18944, 152064, 1e4,
                                qkv_bias=True, tie_lm_head=False),
}

WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1", GEOMETRIES["tiny"], 4, 64, 64, 32, 0.0, 0),
    "C2": Workload("C2", GEOMETRIES["qwen3-0.6b"], 64, 512, 512, 256, 1.0, 1),
    "C3": Workload("C3", GEOMETRIES["qwen3-4b"], 128, 256, 1024, 512, 1.0, 2),
    "C4": Workload("C4", GEOMETRIES["qwen3-4b"], 128, 1024, 4096, 1024, 1.0, 3),
    "C5": Workload("C5", GEOMETRIES["qwen2.5-7b"], 64, 512, 2048, 1024, 1.0, 4),
}


def scaled_geometry(base: str, **overrides) -> ModelGeometry:
    """A geometry derived from a named one with some fields replaced (used to
    build reduced-depth / reduced-vocab test cases that keep the real tile shapes)."""
    g = asdict(GEOMETRIES[base])
    g.update(overrides)
    return ModelGeometry(**g)


# ----------------------------------------------------------------------------
# bf16 storage format helpers (a data format, not model arithmetic)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to the nearest bf16 (ties to even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# weights
# ----------------------------------------------------------------------------
LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "bq", "bk", "bv", "q_norm", "k_norm",
                 "wo", "mlp_norm", "w_gate", "w_up", "w_down")


def layer_tensor_shapes(g: ModelGeometry) -> Dict[str, Tuple[int, ...]]:
    d, hq, hkv, hd, f = g.d_model, g.n_q_heads, g.n_kv_heads, g.head_dim, g.ffn_dim
    shapes = {
        "attn_norm": (d,), "wq": (hq * hd, d), "wk": (hkv * hd, d), "wv": (hkv * hd, d),
        "wo": (d, hq * hd), "mlp_norm": (d,), "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
    }
    if g.qkv_bias:
        shapes.update({"bq": (hq * hd,), "bk": (hkv * hd,), "bv": (hkv * hd,)})
    if g.qk_norm:
        shapes.update({"q_norm": (hd,), "k_norm": (hd,)})
    return shapes


def _is_gain(name: str) -> bool:
    return name.endswith("norm")


def make_weights(g: ModelGeometry, seed: int, std: float = 0.02) -> Dict[str, object]:
    """Random-init weights as host numpy arrays.

    Matrices, embeddings, LM head and QKV biases are N(0, std); every RMSNorm
    gain (layer norms, final norm, per-head q/k norms) is 1.  For bf16
    geometries matrices and biases are rounded to bf16 and returned as uint16
    bit patterns; gains stay fp32.  Returns
    {"embed", "final_norm", "lm_head", "layers": [ {name: array} ]}.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    bf16 = g.weight_dtype == WEIGHT_BF16

    def draw(shape):
        w = (rng.standard_normal(shape, dtype=np.float32) * np.float32(std))
        return f32_to_bf16_bits(w) if bf16 else w

    out: Dict[str, object] = {"embed": draw((g.vocab, g.d_model))}
    layers: List[Dict[str, np.ndarray]] = []
    for _ in range(g.n_layers):
        lw: Dict[str, np.ndarray] = {}
        for name, shape in layer_tensor_shapes(g).items():
            lw[name] = np.ones(shape, dtype=np.float32) if _is_gain(name) else draw(shape)
        layers.append(lw)
    out["layers"] = layers
    out["final_norm"] = np.ones((g.d_model,), dtype=np.float32)
    out["lm_head"] = out["embed"] if g.tie_lm_head else draw((g.vocab, g.d_model))
    return out


def make_weights_torch(g: ModelGeometry, seed: int, device, std: float = 0.02):
    """Same recipe drawn with torch's generator on `device` (fast path for the
    multi-billion-parameter geometries).  Returns the same structure holding
    torch tensors: bf16 (or fp32) matrices, fp32 gains.  The streams differ
    from make_weights(); a test uses one or the other for both sides."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    wdt = torch.bfloat16 if g.weight_dtype == WEIGHT_BF16 else torch.float32

    def draw(shape):
        w = torch.empty(shape, dtype=torch.float32, device=device)
        w.normal_(0.0, std, generator=gen)
        return w.to(wdt)

    out = {"embed": draw((g.vocab, g.d_model))}
    layers = []
    for _ in range(g.n_layers):
        lw = {}
        for name, shape in layer_tensor_shapes(g).items():
            lw[name] = (torch.ones(shape, dtype=torch.float32, device=device)
                        if _is_gain(name) else draw(shape))
        layers.append(lw)
    out["layers"] = layers
    out["final_norm"] = torch.ones((g.d_model,), dtype=torch.float32, device=device)
    out["lm_head"] = out["embed"] if g.tie_lm_head else draw((g.vocab, g.d_model))
    return out


def weights_to_host_numpy(w) -> Dict[str, object]:
    """torch weights (any device) -> the make_weights() host format
    (uint16 bit patterns for bf16 tensors, fp32 arrays otherwise)."""
    import torch

    def conv(t):
        t = t.detach().cpu().contiguous()
        if t.dtype == torch.bfloat16:
            return t.view(torch.int16).numpy().view(np.uint16)
        return t.numpy()

    out = {"embed": conv(w["embed"]), "final_norm": conv(w["final_norm"])}
    out["lm_head"] = out["embed"] if w["lm_head"] is w["embed"] else conv(w["lm_head"])
    out["layers"] = [{k: conv(v) for k, v in lw.items()} for lw in w["layers"]]
    return out


# ----------------------------------------------------------------------------
# prompts, forced tokens, page orders, game outcomes
# ----------------------------------------------------------------------------
def make_prompts(vocab: int, batch: int, lo: int, hi: int, seed: int) -> List[np.ndarray]:
    """`batch` prompts with lengths uniform in [lo, hi] and ids uniform in [0, vocab)."""
    rng = np.random.Generator(np.random.PCG64(seed + 1000))
    lens = rng.integers(lo, hi + 1, size=batch)
    return [rng.integers(0, vocab, size=int(n)).astype(np.int32) for n in lens]


def make_forced_tokens(vocab: int, batch: int, steps: int, seed: int) -> np.ndarray:
    """[steps, batch] uniform token ids used to teacher-force a decode run."""
    rng = np.random.Generator(np.random.PCG64(seed + 2000))
    return rng.integers(0, vocab, size=(steps, batch)).astype(np.int32)


def make_page_order(n_pages: int, seed: int) -> np.ndarray:
    """A seeded permutation of physical page ids: the order in which the pool
    hands pages out, so that a sequence's pages are scattered in memory."""
    rng = np.random.Generator(np.random.PCG64(seed + 3000))
    return rng.permutation(n_pages).astype(np.int32)


def make_game_outcomes(n_games: int, n_traj: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """(game_id[n_traj], R0[n_traj]) with R0 in {-1, 0, 1}: terminal rewards of
    player 0 for a batch of finished zero-sum games (Sec. 3, formulation)."""
    rng = np.random.Generator(np.random.PCG64(seed + 4000))
    return (rng.integers(0, n_games, size=n_traj).astype(np.int32),
            rng.integers(-1, 2, size=n_traj).astype(np.float64))


def make_uniform_noise_free_logits(batch: int, vocab: int, seed: int, scale: float = 1.0) -> np.ndarray:
    """Synthetic logits ~ N(0, scale) for sampler-only tests."""
    rng = np.random.Generator(np.random.PCG64(seed + 5000))
    return (rng.standard_normal((batch, vocab)) * scale).astype(np.float32)
