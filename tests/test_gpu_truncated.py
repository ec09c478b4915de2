"""GPU parity of spiral_sample_truncated (top-k / top-p Gumbel-max) against oracle/truncated.py.
The threshold is index / ordering work on fp32 values and is compared bit for bit wherever the
oracle's running sum does not come within 1e-8 of the cut (the kernel adds 2^-45 fixed-point masses,
the oracle float64); tokens are compared where the top-1/top-2 margin inside the keep set exceeds 0.1."""
import numpy as np
import pytest

from oracle import sampling as osamp
from oracle import truncated as otr

pytestmark = pytest.mark.gpu
MARGIN = 0.1
SLACK = 1e-8


@pytest.fixture(scope="module")
def sb():
    import torch
    assert torch.cuda.is_available()
    from paper_2506_24119_amd import binding
    binding.load_library()
    return binding


def _run(sb, logits, T, k, p, seed, ids, steps, noise=None, want_tau=True, ws=False):
    """ws: the multi-kernel path on a workspace (spiral_sample_truncated_ws) instead of the single kernel"""
    import torch
    B, V = logits.shape
    lg = torch.from_numpy(logits).cuda()
    out = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    tau = torch.zeros(B, dtype=torch.float32, device="cuda") if want_tau else None
    nz = None if noise is None else torch.from_numpy(noise).cuda()
    if ws:
        need = sb.spiral_sample_truncated_workspace_bytes(B, V)
        assert need > 0
        work = torch.full((need,), 0xA5, dtype=torch.uint8, device="cuda")     # the call may not rely on its contents
        sb.spiral_sample_truncated_ws(lg, B, V, T, k, p, seed, ids, steps, nz, out, tau, work, need)
    else:
        sb.spiral_sample_truncated(lg, B, V, T, k, p, seed, ids, steps, nz, out, tau)
    torch.cuda.synchronize()
    return out.cpu().numpy(), (tau.cpu().numpy() if want_tau else None)


SETTINGS = [(0.6, 0, 0.95),        # the paper's evaluation setting
            (1.0, 50, 1.0), (0.8, 20, 0.9), (1.0, 0, 0.5), (1.3, 1, 1.0), (0.6, 3, 0.999), (1.0, 0, 1e-6)]


@pytest.mark.parametrize("V", [151936, 40000, 1000, 7])
@pytest.mark.parametrize("T,k,p", SETTINGS)
def test_threshold_and_token_match_oracle(sb, V, T, k, p):
    rng = np.random.default_rng(V + int(1000 * T) + k)
    B = 9
    logits = (rng.normal(size=(B, V)) * rng.choice([0.3, 1.0, 3.0], size=(B, 1))).astype(np.float32)
    logits[1] = np.round(logits[1] * 2) / 2                     # many equal scores
    p32 = float(np.float32(p))
    ids = np.arange(B, dtype=np.int32) + 3
    steps = np.arange(B, dtype=np.int32) * 7
    seed = 99
    noise = np.stack([osamp.gumbel_noise(seed, int(ids[b]), int(steps[b]), V) for b in range(B)])
    single = {}
    for nz, ws in ((noise, False), (None, False), (noise, True), (None, True)):   # noise buffer / generated stream; both paths
        got_tok, got_tau = _run(sb, logits, T, k, p32, seed, ids, steps, noise=nz, ws=ws)
        if ws:          # the same integers summed in another grouping: every row equal, the undecidable ones included
            assert np.array_equal(got_tau, single[nz is None][1]) and np.array_equal(got_tok, single[nz is None][0])
        else:
            single[nz is None] = (got_tok, got_tau)
        decided = compared = 0
        for b in range(B):
            tok, margin, tau, slack = otr.sample_row(logits[b], T, k, p32, noise[b])
            if slack < SLACK:
                continue
            decided += 1
            assert got_tau[b] == tau, (b, got_tau[b], tau, slack)
            if margin > MARGIN:
                compared += 1
                assert got_tok[b] == tok, (b, got_tok[b], tok, margin)
            else:                                                # still a member of the keep set
                assert otr.scaled(logits[b], T)[got_tok[b]] >= tau
        assert decided >= B - 3


def test_no_truncation_equals_plain_sampler_and_greedy(sb):
    import torch
    rng = np.random.default_rng(5)
    B, V = 6, 5000
    logits = rng.normal(size=(B, V)).astype(np.float32)
    ids = np.arange(B, dtype=np.int32); steps = np.full(B, 4, dtype=np.int32)
    lg = torch.from_numpy(logits).cuda()
    plain = torch.empty(B, dtype=torch.int32, device="cuda")
    sb.spiral_sample(lg, B, V, 0.7, 11, ids, steps, None, plain)
    for k in (0, -1, V, V + 1):
        got, tau = _run(sb, logits, 0.7, k, 1.0, 11, ids, steps)
        assert np.array_equal(got, plain.cpu().numpy()) and np.isneginf(tau).all()
        got, _ = _run(sb, logits, 0.7, k, 1.0, 11, ids, steps, want_tau=False)
        assert np.array_equal(got, plain.cpu().numpy())
    got, _ = _run(sb, logits, 0.0, 5, 0.3, 11, ids, steps, want_tau=False)         # temperature 0: greedy whatever the cut
    assert np.array_equal(got, logits.argmax(axis=1))
    got, _ = _run(sb, logits, 0.7, 1, 1.0, 11, ids, steps)
    assert np.array_equal(got, logits.argmax(axis=1))


def test_ties_are_kept_together_and_results_are_reproducible(sb):
    V = 4096
    row = np.zeros(V, dtype=np.float32)
    row[100:110] = 2.0                                           # ten tokens tie for the top
    row[7] = 1.0
    logits = np.stack([row, row])
    ids = np.array([0, 1], dtype=np.int32); steps = np.array([0, 0], dtype=np.int32)
    tok, tau = _run(sb, logits, 1.0, 3, 1.0, 1, ids, steps)     # k = 3 falls inside the tie group: all ten stay
    assert (tau == 2.0).all() and all(100 <= t < 110 for t in tok)
    seen = set()
    for s in range(40):
        t, _ = _run(sb, logits[:1], 1.0, 3, 1.0, 1, ids[:1], np.array([s], dtype=np.int32))
        seen.add(int(t[0]))
    assert seen <= set(range(100, 110)) and len(seen) >= 6       # the draw really ranges over the tie group
    a = _run(sb, logits, 0.9, 0, 0.7, 5, ids, steps)
    b = _run(sb, logits, 0.9, 0, 0.7, 5, ids, steps)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_large_batch_and_argument_errors(sb):
    import torch
    rng = np.random.default_rng(6)
    B, V = 131, 777                                              # more rows than one launch carries keys for
    logits = rng.normal(size=(B, V)).astype(np.float32)
    ids = np.arange(B, dtype=np.int32); steps = np.zeros(B, dtype=np.int32)
    got_tok, got_tau = _run(sb, logits, 0.6, 0, float(np.float32(0.95)), 3, ids, steps)
    for b in (0, 127, 128, 130):
        g = osamp.gumbel_noise(3, b, 0, V)
        tok, margin, tau, slack = otr.sample_row(logits[b], 0.6, 0, float(np.float32(0.95)), g)
        if slack >= SLACK:
            assert got_tau[b] == tau
            if margin > MARGIN:
                assert got_tok[b] == tok
    lg = torch.from_numpy(logits).cuda()
    out = torch.empty(B, dtype=torch.int32, device="cuda")
    for bad_p in (0.0, -0.5, 1.5, float("nan")):
        with pytest.raises(sb.SpiralError) as e:
            sb.spiral_sample_truncated(lg, B, V, 1.0, 0, bad_p, 0, ids, steps, None, out, None)
        assert e.value.code == sb.SPIRAL_ERR_INVALID_ARG
    with pytest.raises(sb.SpiralError):
        sb.spiral_sample_truncated(lg, B, V, 1.0, 5, 0.9, 0, None, None, None, out, None)


def test_workspace_path_large_batch_crowded_rows_and_errors(sb):
    """More rows than one launch carries keys for; rows whose scores crowd around the cut (all equal, two values, a
    narrow spread) overflow the candidate list and are done by the single kernel inside the same call."""
    import torch
    rng = np.random.default_rng(16)
    B, V = 131, 20000
    logits = rng.normal(size=(B, V)).astype(np.float32)
    logits[5] = 1.25                                             # every score equal
    logits[6] = np.where(rng.random(V) < 0.5, 0.5, -0.5)        # two values
    logits[7] = (rng.normal(size=V) * 1e-3).astype(np.float32)  # 20000 scores inside a few bins
    logits[129] = 3.0
    logits[8, ::17] = -np.inf                                   # masked-out tokens
    ids = np.arange(B, dtype=np.int32); steps = np.arange(B, dtype=np.int32)
    for T, k, p in ((0.6, 0, 0.95), (1.0, 40, 1.0), (0.8, 9000, 0.9), (1.0, 12000, 1.0)):
        p32 = float(np.float32(p))
        a = _run(sb, logits, T, k, p32, 3, ids, steps)
        b = _run(sb, logits, T, k, p32, 3, ids, steps, ws=True)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]), (T, k, p)
        for r in (0, 5, 6, 7, 8, 127, 128, 129, 130):
            g = osamp.gumbel_noise(3, r, int(steps[r]), V)
            tok, margin, tau, slack = otr.sample_row(logits[r], T, k, p32, g)
            if slack >= SLACK:
                assert b[1][r] == tau, (T, k, p, r)
                if margin > MARGIN:
                    assert b[0][r] == tok
    lg = torch.from_numpy(logits).cuda()
    out = torch.empty(B, dtype=torch.int32, device="cuda")
    need = sb.spiral_sample_truncated_workspace_bytes(B, V)
    work = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
    for bad in ((None, need), (work, need - 1), (work[1:], need)):                # null, too small, misaligned
        with pytest.raises(sb.SpiralError) as e:
            sb.spiral_sample_truncated_ws(lg, B, V, 0.6, 0, 0.95, 0, ids, steps, None, out, None, bad[0], bad[1])
        assert e.value.code == sb.SPIRAL_ERR_INVALID_ARG
    assert sb.spiral_sample_truncated_workspace_bytes(0, V) == 0 and sb.spiral_sample_truncated_workspace_bytes(B, 0) == 0
