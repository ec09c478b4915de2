"""Pins for oracle/decoder.py: closed forms, special cases, invariants and an
independent library implementation.  None of these re-types the oracle's own
formulas as the expected value."""
import numpy as np
import pytest
import torch

from oracle import decoder as od
from paper_2506_24119_amd import inputs as si


def _rand_gains(w, rng):
    """Non-trivial gains so that a misplaced or dropped gain is visible."""
    for lw in w["layers"]:
        for k in lw:
            if k.endswith("norm"):
                lw[k] = (1.0 + 0.3 * rng.standard_normal(lw[k].shape)).astype(np.float32)
    w["final_norm"] = (1.0 + 0.3 * rng.standard_normal(w["final_norm"].shape)).astype(np.float32)
    return w


SMALL_QK = si.ModelGeometry("small-qk", 3, 48, 6, 2, 16, 80, 97, 1e4, qk_norm=True,
                            weight_dtype=si.WEIGHT_FP32)
SMALL_BIAS = si.ModelGeometry("small-bias", 2, 48, 6, 3, 8, 64, 61, 5e5, qkv_bias=True,
                              tie_lm_head=False, weight_dtype=si.WEIGHT_FP32)


# ---------------------------------------------------------------- storage
def test_bf16_widen_exact_patterns():
    bits = np.array([0x3F80, 0xC000, 0x0000, 0x3E80, 0x4049, 0xBDCD], dtype=np.uint16)
    # 1.0, -2.0, 0, 0.25, 3.140625, -0.10009765625 : hand-decoded sign/exponent/7-bit mantissa
    want = np.array([1.0, -2.0, 0.0, 0.25, 3.140625, -0.10009765625])
    assert np.array_equal(od.widen(bits), want)


def test_bf16_rounding_in_inputs_is_nearest_even():
    # 1 + 2^-8 is exactly half-way between bf16 neighbours 1.0 and 1+2^-7: ties to even -> 1.0
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    got = si.bf16_bits_to_f32(si.f32_to_bf16_bits(x))
    assert np.array_equal(got, np.array([1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7], dtype=np.float32))
    # and matches torch's conversion on random data
    r = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    t = torch.from_numpy(r).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(si.f32_to_bf16_bits(r), t)


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_matches_library_and_unit_rms():
    rng = np.random.default_rng(1)
    v = rng.standard_normal((5, 33))
    g = rng.standard_normal(33)
    want = torch.nn.functional.rms_norm(torch.from_numpy(v), (33,), torch.from_numpy(g), 1e-6).numpy()
    np.testing.assert_allclose(od.rmsnorm(v, g, 1e-6), want, rtol=1e-12, atol=1e-14)
    out = od.rmsnorm(v, np.ones(33), 0.0)
    np.testing.assert_allclose(np.sqrt((out ** 2).mean(-1)), 1.0, rtol=1e-12)
    # eps sits inside the square root next to the mean square: a zero vector maps to zero, not NaN
    assert np.array_equal(od.rmsnorm(np.zeros((1, 4)), np.ones(4), 1e-6), np.zeros((1, 4)))
    # scale invariance (up to eps)
    np.testing.assert_allclose(od.rmsnorm(7.0 * v, g, 0.0), od.rmsnorm(v, g, 0.0), rtol=1e-12)


# ---------------------------------------------------------------- RoPE
def test_rope_closed_forms():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((6, 3, 16))
    pos = np.array([0, 1, 2, 5, 100, 4095])
    y = od.rope(x, pos, 1e4)
    assert np.array_equal(y[0], x[0])                                   # position 0 is the identity
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    # hd = 2: a plain 2x2 rotation by pos * theta^0 = pos radians
    v = np.array([[[1.0, 0.0]], [[0.3, -0.7]]])
    p = np.array([3, 11])
    r = od.rope(v, p, 123.0)
    for i in range(2):
        c, s = np.cos(p[i]), np.sin(p[i])
        np.testing.assert_allclose(r[i, 0], np.array([[c, -s], [s, c]]) @ v[i, 0], rtol=1e-12, atol=1e-15)
    # pair j uses frequency theta^(-2j/hd): with hd = 4, theta = 100 the second pair turns by pos/10
    v4 = np.array([[[0.0, 1.0, 0.0, 0.0]]])
    r4 = od.rope(v4, np.array([5]), 100.0)[0, 0]
    np.testing.assert_allclose(r4, [0.0, np.cos(0.5), 0.0, np.sin(0.5)], atol=1e-15)


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(3)
    q = rng.standard_normal((1, 1, 32))
    k = rng.standard_normal((1, 1, 32))
    def score(m, n):
        return float(np.sum(od.rope(q, np.array([m]), 1e6) * od.rope(k, np.array([n]), 1e6)))
    assert abs(score(7, 3) - score(1007, 1003)) < 1e-9
    assert abs(score(7, 3) - score(4, 0)) < 1e-9
    assert abs(score(7, 3) - score(3, 7)) > 1e-3          # not symmetric in (m, n)


# ---------------------------------------------------------------- SwiGLU
def test_silu_properties_and_library():
    z = np.linspace(-9, 9, 37)
    assert od.silu(np.zeros(1))[0] == 0.0
    np.testing.assert_allclose(od.silu(z) - od.silu(-z), z, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(od.silu(z), torch.nn.functional.silu(torch.from_numpy(z)).numpy(), rtol=1e-12)


# ---------------------------------------------------------------- attention
def test_attention_special_cases():
    rng = np.random.default_rng(4)
    T, hq, hkv, hd = 9, 4, 2, 8
    q = rng.standard_normal((T, hq, hd))
    k = rng.standard_normal((T, hkv, hd))
    v = rng.standard_normal((T, hkv, hd))
    o = od.causal_attention(q, k, v)
    # the first position sees only itself: output is V_0 of its kv head
    for h in range(hq):
        np.testing.assert_allclose(o[0, h], v[0, h // 2], rtol=1e-13)
    # equal keys => uniform weights => running mean of V
    keq = np.broadcast_to(k[:1], k.shape).copy()
    oe = od.causal_attention(q, keq, v)
    run_mean = np.cumsum(v, axis=0) / np.arange(1, T + 1)[:, None, None]
    for h in range(hq):
        np.testing.assert_allclose(oe[:, h], run_mean[:, h // 2], rtol=1e-12)
    # a query orthogonal... adding a per-row constant to all scores changes nothing:
    # K + c*q_dir shifts every score of a row by the same amount only if all keys get the same shift
    shift = rng.standard_normal((1, hkv, hd))
    o2 = od.causal_attention(q, k + shift, v)
    np.testing.assert_allclose(o2, o, rtol=1e-9, atol=1e-12)
    # future positions never leak: changing K,V after position t leaves outputs up to t alone
    k3, v3 = k.copy(), v.copy()
    k3[5:] += 10.0
    v3[5:] -= 3.0
    np.testing.assert_allclose(od.causal_attention(q, k3, v3)[:5], o[:5], rtol=1e-13)


@pytest.mark.parametrize("hq,hkv", [(4, 4), (6, 2), (7, 1)])
def test_attention_matches_library_sdpa(hq, hkv):
    rng = np.random.default_rng(5)
    T, hd = 11, 16
    q = rng.standard_normal((T, hq, hd))
    k = rng.standard_normal((T, hkv, hd))
    v = rng.standard_normal((T, hkv, hd))
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2)[None].repeat_interleave(hq // hkv, dim=1)
    tv = torch.from_numpy(v).permute(1, 0, 2)[None].repeat_interleave(hq // hkv, dim=1)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(od.causal_attention(q, k, v), want, rtol=1e-10, atol=1e-12)
    # the single-query form equals the last row of the full form
    np.testing.assert_allclose(od.single_query_attention(q[-1], k, v), want[-1], rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- whole model
def _hf_logits(g, w, tokens):
    tr = pytest.importorskip("transformers")
    common = dict(vocab_size=g.vocab, hidden_size=g.d_model, intermediate_size=g.ffn_dim,
                  num_hidden_layers=g.n_layers, num_attention_heads=g.n_q_heads,
                  num_key_value_heads=g.n_kv_heads, rope_theta=g.rope_theta, rms_norm_eps=g.rms_eps,
                  tie_word_embeddings=g.tie_lm_head, max_position_embeddings=512,
                  attn_implementation="eager", use_sliding_window=False)
    if g.qk_norm:
        cfg = tr.Qwen3Config(head_dim=g.head_dim, attention_bias=False, **common)
        model = tr.Qwen3ForCausalLM(cfg)
    else:
        assert g.head_dim * g.n_q_heads == g.d_model
        cfg = tr.Qwen2Config(**common)
        model = tr.Qwen2ForCausalLM(cfg)
    model = model.double().eval()
    sd = {}
    T = lambda a: torch.from_numpy(np.asarray(od.widen(a)))
    sd["model.embed_tokens.weight"] = T(w["embed"])
    sd["model.norm.weight"] = T(w["final_norm"])
    sd["lm_head.weight"] = T(w["lm_head"])
    names = {"attn_norm": "input_layernorm.weight", "mlp_norm": "post_attention_layernorm.weight",
             "wq": "self_attn.q_proj.weight", "wk": "self_attn.k_proj.weight", "wv": "self_attn.v_proj.weight",
             "bq": "self_attn.q_proj.bias", "bk": "self_attn.k_proj.bias", "bv": "self_attn.v_proj.bias",
             "q_norm": "self_attn.q_norm.weight", "k_norm": "self_attn.k_norm.weight",
             "wo": "self_attn.o_proj.weight", "w_gate": "mlp.gate_proj.weight", "w_up": "mlp.up_proj.weight",
             "w_down": "mlp.down_proj.weight"}
    for i, lw in enumerate(w["layers"]):
        for k, a in lw.items():
            sd[f"model.layers.{i}.{names[k]}"] = T(a)
    missing, unexpected = model.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in m or "lm_head" in m for m in missing), (missing, unexpected)
    with torch.no_grad():
        return model(torch.from_numpy(np.asarray(tokens, dtype=np.int64))[None]).logits[0].numpy()


@pytest.mark.parametrize("g", [SMALL_QK, SMALL_BIAS], ids=lambda g: g.name)
def test_forward_full_matches_independent_library_model(g):
    """The same weights loaded into the transformers library's reference
    decoder of the model family the paper trains (Qwen3: per-head q/k RMSNorm,
    tied head; Qwen2.5 / R1-Distill: QKV bias, untied head) give the same logits."""
    rng = np.random.default_rng(6)
    w = _rand_gains(si.make_weights(g, seed=11, std=0.2), rng)
    tokens = rng.integers(0, g.vocab, size=13)
    want = _hf_logits(g, w, tokens)
    got = od.forward_full(g, w, tokens)
    # the library builds its rotary cos/sin tables in fp32 whatever the model dtype, which
    # bounds the agreement at ~1e-6; any structural mistake shows up at O(1)
    assert np.abs(got - want).max() <= 2e-5 * np.abs(want).max()


def test_zero_layer_matrices_reduce_to_norm_times_head():
    g = SMALL_QK
    w = si.make_weights(g, seed=3, std=0.5)
    for lw in w["layers"]:
        for k in ("wo", "w_down"):
            lw[k] = np.zeros_like(lw[k])
    tokens = np.array([5, 9, 5, 0])
    got = od.forward_full(g, w, tokens)
    E = w["embed"].astype(np.float64)
    for i, t in enumerate(tokens):
        e = E[t]
        hand = (e / np.sqrt((e * e).sum() / g.d_model + g.rms_eps)) @ E.T
        np.testing.assert_allclose(got[i], hand, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("g", [SMALL_QK, SMALL_BIAS, si.GEOMETRIES["tiny"]], ids=lambda g: g.name)
def test_cached_decode_equals_full_recompute(g):
    """KV-cached decode logits equal full-sequence recompute logits."""
    rng = np.random.default_rng(7)
    w = _rand_gains(si.make_weights(g, seed=5, std=0.1 if g.name != "tiny" else 0.02), rng)
    tokens = rng.integers(0, g.vocab, size=24)
    full = od.forward_full(g, w, tokens)
    dec = od.CachedDecoder(g, w)
    got = [dec.prefill(tokens[:9])]
    for t in tokens[9:]:
        got.append(dec.step(int(t)))
    got = np.stack(got)
    scale = np.abs(full).max()
    assert np.abs(got - full[8:]).max() <= 1e-10 * scale
    # chunked prefill (append onto an existing history) gives the same state
    dec2 = od.CachedDecoder(g, w)
    dec2.prefill(tokens[:4])
    l2 = dec2.prefill(tokens[4:9])
    assert np.abs(l2 - full[8]).max() <= 1e-10 * scale


def test_logits_at_selects_rows_and_prefix_independence():
    g = SMALL_QK
    w = si.make_weights(g, seed=8, std=0.2)
    rng = np.random.default_rng(8)
    tokens = rng.integers(0, g.vocab, size=10)
    full = od.forward_full(g, w, tokens)
    np.testing.assert_array_equal(od.forward_full(g, w, tokens, logits_at=[2, 9]), full[[2, 9]])
    # logits at t depend only on tokens 0..t
    np.testing.assert_allclose(od.forward_full(g, w, tokens[:6])[5], full[5], rtol=1e-12, atol=1e-13)


def test_forward_full_many_equals_per_sequence_calls():
    g = SMALL_BIAS
    w = si.make_weights(g, seed=9, std=0.2)
    rng = np.random.default_rng(9)
    seqs = [rng.integers(0, g.vocab, size=n) for n in (7, 12, 1)]
    at = [[3, 6], [11], [0]]
    many = od.forward_full_many(g, w, seqs, at)
    for s_, a_, m_ in zip(seqs, at, many):
        np.testing.assert_array_equal(m_, od.forward_full(g, w, s_, logits_at=a_))


def test_fp32_variant_tracks_fp64():
    g = si.GEOMETRIES["tiny"]
    w = si.make_weights(g, seed=0)
    tokens = si.make_prompts(g.vocab, 1, 32, 32, 0)[0]
    a = od.forward_full(g, w, tokens, logits_at=[31])
    b = od.forward_full(g, w, tokens, logits_at=[31], dtype=np.float32)
    assert b.dtype == np.float32
    assert np.abs(a - b).max() <= 1e-4 * a.std()
