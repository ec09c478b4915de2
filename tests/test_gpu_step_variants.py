"""GPU tests of the decode step's variants and of its contract: the step fused with the sampler against the two
separate calls and against the oracle, independence from workspace contents, the saturation counter, and the
roll-back of a call whose launches fail part-way (forced from the host)."""
import numpy as np
import pytest

from oracle import decoder as od
from oracle import sampling as osamp
from paper_2506_24119_amd import inputs as si

pytestmark = pytest.mark.gpu

LOGIT_TOL = 3e-2
MARGIN = 0.1

G_FUSED = {
    # 4 query heads per kv head, per-head q/k norm; vocabulary of 16 full 128-column tiles
    "g4": si.ModelGeometry("g4-qknorm", 2, 256, 8, 2, 128, 640, 2048, 1e6, qk_norm=True),
    # a vocabulary whose last tile holds 16 of 128 columns, untied head, QKV bias
    "g2-ragged-vocab": si.ModelGeometry("g2-ragged-vocab", 2, 128, 4, 2, 64, 384, 5008, 1e4, qkv_bias=True, tie_lm_head=False),
}


@pytest.fixture(scope="module")
def sb():
    import torch
    assert torch.cuda.is_available()
    from paper_2506_24119_amd import binding
    binding.load_library()
    return binding


def _session(sb, g, w, B, max_ctx=160, tune=None, page_seed=5):
    n_pages = B * ((max_ctx + 15) // 16) + 2
    return sb.Session(g, sb.weights_to_device(w), n_pages, B, (max_ctx + 15) // 16, 1024, max_ctx,
                      page_order=si.make_page_order(n_pages, page_seed), tune=tune)


@pytest.mark.parametrize("name", list(G_FUSED))
@pytest.mark.parametrize("T", [1.0, 0.0])
def test_fused_sample_step_equals_separate_calls_and_oracle(sb, name, T):
    import torch
    g = G_FUSED[name]
    w = si.make_weights(g, seed=31)
    B, steps, seed = 7, 12, 777
    prompts = si.make_prompts(g.vocab, B, 1, 60, seed=32)
    forced = si.make_forced_tokens(g.vocab, B, steps, seed=33)
    ids = np.arange(B, dtype=np.int32)
    a, b = _session(sb, g, w, B), _session(sb, g, w, B)
    la = a.prefill(ids, prompts)
    b.prefill(ids, prompts)
    tok_a = torch.empty(B, dtype=torch.int32, device="cuda")
    tok_b = torch.empty(B, dtype=torch.int32, device="cuda")
    got = []
    for k in range(steps):
        tin = torch.from_numpy(np.ascontiguousarray(forced[k])).cuda()
        st = np.full(B, k + 1, dtype=np.int32)
        a.decode_step(ids, tin, la)
        a.sample(la, T, seed, ids, st, tok_a)
        b.decode_sample_step(ids, tin, T, seed, st, tok_b)
        assert torch.equal(tok_a, tok_b), f"step {k}: {tok_a.tolist()} vs {tok_b.tolist()}"
        got.append(tok_b.cpu().numpy().copy())
    # and against the oracle's draw from the oracle's logits, wherever its decision is clear
    compared = 0
    for s in range(B):
        toks = np.concatenate([prompts[s], forced[:, s]]).astype(np.int64)
        want = od.forward_full(g, w, toks, logits_at=np.arange(len(prompts[s]), len(toks)))
        for k in range(steps):
            noise = osamp.gumbel_noise(seed, s, k + 1, g.vocab) if T > 0 else None
            t, margin = osamp.sample_row(want[k], T, noise)
            if margin > MARGIN:
                compared += 1
                assert got[k][s] == t, (name, T, s, k, got[k][s], t, margin)
    assert compared > steps
    # free-running: the output buffer is the next step's input buffer
    for k in range(4):
        st = np.full(B, steps + 1 + k, dtype=np.int32)
        a.decode_step(ids, tok_a, la)
        a.sample(la, T, seed, ids, st, tok_a)
        b.decode_sample_step(ids, tok_b, T, seed, st, tok_b)
        assert torch.equal(tok_a, tok_b)
    assert a.saturation_count() == 0 and b.saturation_count() == 0
    a.close(); b.close()


def test_fused_step_rejects_what_it_cannot_run(sb):
    import torch
    g = si.ModelGeometry("odd-vocab", 2, 128, 4, 2, 64, 384, 1000, 1e4)         # vocab % 16 != 0
    w = si.make_weights(g, seed=34)
    s = _session(sb, g, w, 2)
    s.prefill([0, 1], si.make_prompts(g.vocab, 2, 5, 9, seed=35))
    tok = torch.zeros(2, dtype=torch.int32, device="cuda")
    with pytest.raises(sb.SpiralError) as e:
        s.decode_sample_step(np.arange(2, dtype=np.int32), tok, 1.0, 1, np.zeros(2, dtype=np.int32), tok)
    assert e.value.code == sb.SPIRAL_ERR_SHAPE
    assert sb.spiral_seq_len(s.pool, 0) + sb.spiral_seq_len(s.pool, 1) == sum(len(p) for p in si.make_prompts(g.vocab, 2, 5, 9, seed=35))
    g2 = G_FUSED["g4"]
    s2 = _session(sb, g2, si.make_weights(g2, seed=31), 2)
    s2.prefill([0, 1], si.make_prompts(g2.vocab, 2, 5, 9, seed=35))
    for bad_T, steps in ((-1.0, np.zeros(2, dtype=np.int32)), (float("nan"), np.zeros(2, dtype=np.int32)), (1.0, None),
                         (1.0, np.array([0, -3], dtype=np.int32))):
        with pytest.raises(sb.SpiralError) as e:
            s2.decode_sample_step(np.arange(2, dtype=np.int32), tok, bad_T, 1, steps, tok)
        assert e.value.code == sb.SPIRAL_ERR_INVALID_ARG
    s.close(); s2.close()


def test_workspace_contents_do_not_carry_between_calls(sb):
    """The caller may reuse, clear or scribble over the workspace between calls, and two pools may share one."""
    import torch
    g = G_FUSED["g4"]
    w = si.make_weights(g, seed=36)
    B, steps = 5, 6
    prompts = si.make_prompts(g.vocab, B, 3, 50, seed=37)
    forced = si.make_forced_tokens(g.vocab, B, steps, seed=38)
    ids = np.arange(B, dtype=np.int32)
    clean, dirty, other = _session(sb, g, w, B), _session(sb, g, w, B), _session(sb, g, w, B, page_seed=6)
    other.ws = dirty.ws                                    # two pools, one workspace
    lc, ld = clean.prefill(ids, prompts), dirty.prefill(ids, prompts)
    lo = other.prefill(ids[:3][::-1].copy(), [prompts[2], prompts[1], prompts[0]])
    assert torch.equal(lc, ld)
    for k in range(steps):
        tin = torch.from_numpy(np.ascontiguousarray(forced[k])).cuda()
        dirty.ws.fill_(0xFF if k % 2 else 0)
        other.decode_step(ids[:3][::-1].copy(), tin[:3], lo)          # another pool's ids go through the same workspace
        clean.decode_step(ids, tin, lc)
        dirty.decode_step(ids, tin, ld)
        assert torch.equal(lc, ld), f"step {k}"
    clean.close(); dirty.close(); other.close()


def test_out_of_range_activations_are_counted_and_clamped(sb):
    """Gate/up weights scaled so that SiLU(g) * u leaves the half range: the store saturates at +-65504 (no inf, no
    NaN downstream) and the pool's counter reports it.  With a zero down projection the MLP branch contributes
    nothing either way, so the logits still match the oracle, which never clamps."""
    import torch
    g = G_FUSED["g4"]
    w = si.make_weights(g, seed=39)
    for lw in w["layers"]:
        for name in ("w_gate", "w_up"):
            f = si.bf16_bits_to_f32(lw[name]) * 1500.0
            lw[name] = si.f32_to_bf16_bits(f.astype(np.float32))
        lw["w_down"] = np.zeros_like(lw["w_down"])
    B = 4
    prompts = si.make_prompts(g.vocab, B, 4, 30, seed=40)
    forced = si.make_forced_tokens(g.vocab, B, 3, seed=41)
    ids = np.arange(B, dtype=np.int32)
    s = _session(sb, g, w, B)
    logits = s.prefill(ids, prompts)
    got = [logits.cpu().numpy().copy()]
    after_prefill = s.saturation_count()
    for k in range(3):
        s.decode_step(ids, torch.from_numpy(np.ascontiguousarray(forced[k])).cuda(), logits)
        got.append(logits.cpu().numpy().copy())
    assert after_prefill > 0 and s.saturation_count() > after_prefill
    got = np.stack(got)
    assert np.isfinite(got).all()
    for b in range(B):
        toks = np.concatenate([prompts[b], forced[:, b]]).astype(np.int64)
        want = od.forward_full(g, w, toks, logits_at=np.arange(len(prompts[b]) - 1, len(toks)))
        ratio = np.abs(got[:, b] - want).max(axis=-1) / want.std(axis=-1)
        assert ratio.max() <= LOGIT_TOL, ratio
    s.close()


def test_a_call_that_fails_part_way_is_rolled_back(sb):
    """A launch failure forced from the host in the middle of a step (nothing is launched in its place): lengths,
    page lists and the free list are as before the call, and the sequences go on to decode correctly."""
    import torch
    g = G_FUSED["g4"]
    w = si.make_weights(g, seed=42)
    B = 3
    prompts = [np.resize(p, n) for p, n in zip(si.make_prompts(g.vocab, B, 40, 40, seed=43), (16, 32, 21))]
    forced = si.make_forced_tokens(g.vocab, B, 2, seed=44)
    ids = np.arange(B, dtype=np.int32)
    s = _session(sb, g, w, B)
    logits = s.prefill(ids, prompts)
    free0 = sb.spiral_kv_free_pages(s.pool)
    tin = torch.from_numpy(np.ascontiguousarray(forced[0])).cuda()
    for n in (1, 4, 9):                                         # first layer's QKV, first O projection, second layer
        sb.spiral_model_tune(s.model, f"fail_after={n}")
        with pytest.raises(sb.SpiralError) as e:
            s.decode_step(ids, tin, logits)                     # sequences 0 and 1 would each take a new page
        assert e.value.code == sb.SPIRAL_ERR_HIP
        assert [sb.spiral_seq_len(s.pool, i) for i in range(B)] == [16, 32, 21]
        assert sb.spiral_kv_free_pages(s.pool) == free0
    sb.spiral_model_tune(s.model, "fail_after=2")
    with pytest.raises(sb.SpiralError):
        s.prefill(ids[:1], [np.zeros(20, dtype=np.int32)])      # a failed append of a turn
    assert sb.spiral_seq_len(s.pool, 0) == 16 and sb.spiral_kv_free_pages(s.pool) == free0
    got = []
    for k in range(2):
        s.decode_step(ids, torch.from_numpy(np.ascontiguousarray(forced[k])).cuda(), logits)
        got.append(logits.cpu().numpy().copy())
    assert sb.spiral_kv_free_pages(s.pool) == free0 - 2
    for b in range(B):
        toks = np.concatenate([prompts[b], forced[:, b]]).astype(np.int64)
        want = od.forward_full(g, w, toks, logits_at=np.arange(len(prompts[b]), len(toks)))
        ratio = np.abs(np.stack(got)[:, b] - want).max(axis=-1) / want.std(axis=-1)
        assert ratio.max() <= LOGIT_TOL, (b, ratio)
    s.close()
