"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Tolerances are the stated ones: max |dlogit| <= 3e-2 x per-row logit std (population std
of the oracle's row); greedy / sampled tokens identical wherever the oracle's top-1/top-2 margin of
the (perturbed) scores exceeds 0.1."""
import numpy as np
import pytest

from oracle import decoder as od
from oracle import sampling as osamp
from paper_2506_24119_amd import inputs as si

pytestmark = pytest.mark.gpu

LOGIT_TOL = 3e-2
MARGIN = 0.1


@pytest.fixture(scope="module")
def sb():
    import torch
    assert torch.cuda.is_available()
    from paper_2506_24119_amd import binding
    binding.load_library()
    return binding


def _torch():
    import torch
    return torch


def assert_logits_close(got: np.ndarray, want: np.ndarray, what: str):
    """max |dlogit| <= 3e-2 x per-row std of the oracle's logits."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape and np.isfinite(got).all(), what
    ratio = np.abs(got - want).max(axis=-1) / want.std(axis=-1)
    assert ratio.max() <= LOGIT_TOL, f"{what}: max|dlogit|/std = {ratio.max():.4g} (row {int(ratio.argmax())})"
    return float(ratio.max())


def assert_tokens_match(got: np.ndarray, want: np.ndarray, margins: np.ndarray, what: str):
    sel = margins > MARGIN
    assert np.array_equal(np.asarray(got)[sel], np.asarray(want)[sel]), \
        f"{what}: {np.flatnonzero((np.asarray(got) != np.asarray(want)) & sel)}"
    return int(sel.sum())


def make_session(sb, g, w_host, n_pages, max_seqs, max_blocks, max_rows, max_context, page_seed=None, tune=None):
    order = None if page_seed is None else si.make_page_order(n_pages, page_seed)
    return sb.Session(g, sb.weights_to_device(w_host), n_pages, max_seqs, max_blocks, max_rows, max_context,
                      page_order=order, tune=tune)


def run_teacher_forced(sb, sess, g, prompts, forced, temperature=0.0, seed=0, noise=None):
    """prefill + len(forced) decode steps fed with `forced[k][b]`; returns logits [steps+1, B, V] and
    the tokens spiral_sample picks from each logits matrix."""
    torch = _torch()
    B = len(prompts)
    ids = np.arange(B, dtype=np.int32)
    logits = sess.prefill(ids, prompts)
    out_tok = torch.empty(B, dtype=torch.int32, device=sess.device)
    all_logits, all_tok = [], []

    def pick(k):
        nz = None if noise is None else torch.from_numpy(noise[k]).to(sess.device)
        sess.sample(logits, temperature, seed, ids, np.full(B, k, dtype=np.int32), out_tok, noise=nz)
        all_logits.append(logits.cpu().numpy().copy())
        all_tok.append(out_tok.cpu().numpy().copy())

    pick(0)
    for k in range(forced.shape[0]):
        tin = torch.from_numpy(np.ascontiguousarray(forced[k])).to(sess.device)
        sess.decode_step(ids, tin, logits)
        pick(k + 1)
    torch.cuda.synchronize()
    return np.stack(all_logits), np.stack(all_tok)


def oracle_teacher_forced(g, w_host, prompt, forced_col):
    """Oracle logits after the prompt and after each forced token: one full causal forward."""
    toks = np.concatenate([prompt, forced_col]).astype(np.int64)
    at = np.arange(len(prompt) - 1, len(toks))
    return od.forward_full(g, w_host, toks, logits_at=at)


# ------------------------------------------------------------------------------------------------
# C1: the tiny fp32 configuration, whole workload, greedy
# ------------------------------------------------------------------------------------------------
def test_c1_tiny_greedy_matches_oracle(sb):
    wl = si.WORKLOADS["C1"]
    g = wl.geometry
    w = si.make_weights(g, wl.seed)
    prompts = si.make_prompts(g.vocab, wl.batch, wl.prompt_lo, wl.prompt_hi, wl.seed)
    # the oracle generates greedily; its tokens teacher-force the GPU run
    ref_logits, ref_tok, ref_margin = [], [], []
    for b in range(wl.batch):
        dec = od.CachedDecoder(g, w)
        lg = dec.prefill(prompts[b])
        rows, toks, margins = [], [], []
        for k in range(wl.decode_steps + 1):
            t, m = osamp.sample_row(lg, 0.0)
            rows.append(lg); toks.append(t); margins.append(m)
            if k < wl.decode_steps:
                lg = dec.step(t)
        ref_logits.append(np.stack(rows)); ref_tok.append(toks); ref_margin.append(margins)
    ref_logits = np.stack(ref_logits, axis=1)                   # [steps+1, B, V]
    ref_tok = np.array(ref_tok).T
    ref_margin = np.array(ref_margin).T
    forced = ref_tok[:-1].astype(np.int32)

    sess = make_session(sb, g, w, n_pages=64, max_seqs=wl.batch, max_blocks=8, max_rows=wl.batch * wl.prompt_hi,
                        max_context=wl.prompt_hi + wl.decode_steps + 1, page_seed=1)
    got_logits, got_tok = run_teacher_forced(sb, sess, g, prompts, forced)
    worst = assert_logits_close(got_logits, ref_logits, "C1 logits")
    n = assert_tokens_match(got_tok, ref_tok, ref_margin, "C1 greedy tokens")
    assert n > 0
    print(f"C1: max|dlogit|/std = {worst:.3e}, {n}/{ref_tok.size} tokens compared")
    sess.close()


# ------------------------------------------------------------------------------------------------
# bf16 geometries with the real tile shapes, reduced depth / width so the oracle takes seconds
# ------------------------------------------------------------------------------------------------
SMALL = {
    # Qwen3-4B-like: 4 query heads per kv head, hd 128, per-head q/k norm, tied head
    "g4-qknorm": si.ModelGeometry("g4-qknorm", 2, 256, 8, 2, 128, 640, 2048, 1e6, qk_norm=True),
    # Qwen3-0.6B-like grouping (2 per kv head), three layers
    "g2-qknorm": si.ModelGeometry("g2-qknorm", 3, 128, 4, 2, 128, 384, 1000, 1e6, qk_norm=True),
    # R1-Distill-Qwen-7B-like: 7 query heads per kv head, QKV bias, untied head
    "g7-bias": si.ModelGeometry("g7-bias", 2, 448, 7, 1, 64, 1024, 1536, 1e4, qkv_bias=True, tie_lm_head=False),
    # plain multi-head attention, hd 32
    "g1-mha": si.ModelGeometry("g1-mha", 2, 128, 4, 4, 32, 256, 512, 1e4),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_small_bf16_models_ragged_batch(sb, name):
    g = SMALL[name]
    w = si.make_weights(g, seed=21)
    B, steps = 6, 20
    prompts = si.make_prompts(g.vocab, B, 1, 70, seed=5)       # lengths 1..70: several pages and ragged tails
    prompts[0] = prompts[0][:1]                                 # degenerate: a one-token history
    prompts[1] = np.resize(prompts[1], 16)                      # exactly one full page
    prompts[2] = np.resize(prompts[2], 17)                      # one token into the second page
    forced = si.make_forced_tokens(g.vocab, B, steps, seed=6)
    sess = make_session(sb, g, w, n_pages=64, max_seqs=8, max_blocks=8, max_rows=256, max_context=128, page_seed=2)
    got_logits, got_tok = run_teacher_forced(sb, sess, g, prompts, forced)
    worst, compared = 0.0, 0
    for b in range(B):
        want = oracle_teacher_forced(g, w, prompts[b], forced[:, b])
        worst = max(worst, assert_logits_close(got_logits[:, b], want, f"{name} seq {b}"))
        toks, margins = zip(*[osamp.sample_row(r, 0.0) for r in want])
        compared += assert_tokens_match(got_tok[:, b], np.array(toks), np.array(margins), f"{name} greedy seq {b}")
    print(f"{name}: max|dlogit|/std = {worst:.3e}, {compared} greedy tokens compared")
    assert compared > 0
    sess.close()


def test_long_context_spans_several_attention_chunks(sb):
    """One sequence far longer than a 256-token attention chunk next to a short one."""
    g = SMALL["g4-qknorm"]
    w = si.make_weights(g, seed=22)
    prompts = [si.make_prompts(g.vocab, 1, 700, 700, seed=8)[0], si.make_prompts(g.vocab, 1, 5, 5, seed=9)[0]]
    forced = si.make_forced_tokens(g.vocab, 2, 8, seed=10)
    sess = make_session(sb, g, w, n_pages=80, max_seqs=2, max_blocks=64, max_rows=1024, max_context=1024, page_seed=3)
    got_logits, _ = run_teacher_forced(sb, sess, g, prompts, forced)
    for b in range(2):
        want = oracle_teacher_forced(g, w, prompts[b], forced[:, b])
        assert_logits_close(got_logits[:, b], want, f"long-context seq {b}")
    sess.close()


@pytest.mark.parametrize("tune", ["chunk=1,wgs=7", "chunk=2,wgs=100000", "chunk=64,wgs=3", "chunk=1,wgs=1"])
@pytest.mark.parametrize("name", ["g4-qknorm", "g7-bias"])
def test_decode_attention_launch_shapes(sb, name, tune):
    """The decode attention's page stream with workgroup ranges that cut (row, kv head) pairs at arbitrary
    pages, hold many pairs, hold one page each, or are a single workgroup (spiral_model_tune selects them)."""
    g = SMALL[name]
    w = si.make_weights(g, seed=23)
    B, steps = 5, 18
    prompts = si.make_prompts(g.vocab, B, 1, 90, seed=11)
    prompts[0] = prompts[0][:1]
    prompts[1] = np.resize(prompts[1], 15)                      # the first decode step fills the page exactly
    prompts[2] = np.resize(prompts[2], 16)                      # the first decode step opens a new page
    forced = si.make_forced_tokens(g.vocab, B, steps, seed=12)
    sess = make_session(sb, g, w, n_pages=64, max_seqs=8, max_blocks=8, max_rows=512, max_context=128, page_seed=4, tune=tune)
    got_logits, _ = run_teacher_forced(sb, sess, g, prompts, forced)
    for b in range(B):
        want = oracle_teacher_forced(g, w, prompts[b], forced[:, b])
        assert_logits_close(got_logits[:, b], want, f"{name} [{tune}] seq {b}")
    sess.close()


def test_repacked_weights_give_bit_identical_logits(sb):
    """spiral_model_repack changes where the weight bytes sit and nothing else: prefill (small and large
    row counts), decode and the scoring pass return the same bits with and without it."""
    torch = _torch()
    g = si.ModelGeometry("rp-check", 2, 256, 8, 2, 128, 640, 2000, 1e6, qk_norm=True)
    w = si.make_weights(g, seed=27)
    prompts = si.make_prompts(g.vocab, 6, 3, 200, seed=15)          # ~600 rows: the large-M kernels run too
    forced = si.make_forced_tokens(g.vocab, 6, 5, seed=16)
    outs = []
    for tune in ("frag=0", "frag=1"):
        sess = make_session(sb, g, w, n_pages=96, max_seqs=8, max_blocks=16, max_rows=2048, max_context=256, page_seed=9, tune=tune)
        assert (sess.repacked is not None)
        logits, _ = run_teacher_forced(sb, sess, g, prompts, forced)
        toks = torch.from_numpy(np.concatenate(prompts).astype(np.int32)).cuda()
        tg = torch.from_numpy(np.concatenate([np.concatenate([p[1:], [-1]]) for p in prompts]).astype(np.int32)).cuda()
        lp = torch.empty(toks.numel(), dtype=torch.float32, device="cuda")
        sb.spiral_seq_reset(sess.pool, list(range(6)))
        sb.spiral_score(sess.model, sess.pool, list(range(6)), [len(p) for p in prompts], toks, tg, sess.ws, lp)
        outs.append((logits, lp.cpu().numpy()))
        sess.close()
    assert np.array_equal(outs[0][0], outs[1][0])
    assert np.array_equal(outs[0][1], outs[1][1])


@pytest.mark.parametrize("variant", ["qk_norm", "qkv_bias"])
def test_large_prefill_with_the_qkv_epilogue_in_the_projection(sb, variant):
    """A prefill of ~2,500 rows on a wide q/k/v projection (50 heads of 128) takes the 256 x 256 tiled kernel whose
    epilogue does the bias / per-head norm / RoPE / page append itself; the same call with that fusion switched off
    (spiral_model_tune "fuse_qkv=0": projection, then qkv_post_kernel) must agree to rounding, a page written by the
    epilogue must serve the decode steps that follow, and one sequence is compared with the oracle."""
    g = si.ModelGeometry("wide-qkv", 2, 256, 40, 5, 128, 512, 1500, 1e6,
                         qk_norm=(variant == "qk_norm"), qkv_bias=(variant == "qkv_bias"))
    w = si.make_weights(g, seed=31)
    prompts = si.make_prompts(g.vocab, 6, 300, 520, seed=17)
    prompts[0] = prompts[0][:271]                                   # ends inside a page
    forced = si.make_forced_tokens(g.vocab, 6, 4, seed=18)
    outs = []
    for tune in ("fuse_qkv=1", "fuse_qkv=0"):
        sess = make_session(sb, g, w, n_pages=256, max_seqs=8, max_blocks=40, max_rows=4096, max_context=640, page_seed=12, tune=tune)
        assert sess.repacked is not None
        # which path ran: the post-processing kernel is launched once per layer and decode step, and once per layer
        # more by the prefill when the projection does not do its work
        sb.spiral_profile_begin(sess.model, sb.KERNEL_CLASSES.index("qkv_post"), 1000)
        logits, _ = run_teacher_forced(sb, sess, g, prompts, forced)
        _, n_post = sb.spiral_profile_end(sess.model)
        assert n_post == g.n_layers * (forced.shape[0] + (0 if tune == "fuse_qkv=1" else 1)), (tune, n_post)
        assert sess.saturation_count() == 0
        outs.append(logits)
        sess.close()
    scale = np.abs(outs[1]).max()
    assert np.abs(outs[0] - outs[1]).max() <= 2e-3 * scale         # same arithmetic, another summation order in the norm
    want = oracle_teacher_forced(g, w, prompts[0], forced[:, 0])
    assert_logits_close(outs[0][:, 0], want, f"wide-qkv {variant} seq 0")


# ------------------------------------------------------------------------------------------------
# invariants of the path itself
# ------------------------------------------------------------------------------------------------
def test_page_order_and_batch_composition_do_not_change_logits(sb):
    g = SMALL["g4-qknorm"]
    w = si.make_weights(g, seed=23)
    prompts = si.make_prompts(g.vocab, 4, 20, 60, seed=11)
    forced = si.make_forced_tokens(g.vocab, 4, 6, seed=12)
    runs = []
    for page_seed in (None, 4, 5):
        sess = make_session(sb, g, w, 64, 4, 8, 256, 128, page_seed=page_seed)
        runs.append(run_teacher_forced(sb, sess, g, prompts, forced)[0])
        sess.close()
    assert np.array_equal(runs[0], runs[1]) and np.array_equal(runs[0], runs[2])      # bit-identical
    # a sequence alone gives the same logits as inside the batch
    sess = make_session(sb, g, w, 64, 4, 8, 256, 128, page_seed=6)
    alone, _ = run_teacher_forced(sb, sess, g, prompts[2:3], forced[:, 2:3])
    sess.close()
    scale = np.abs(runs[0][:, 2]).max()
    assert np.abs(alone[:, 0] - runs[0][:, 2]).max() <= 1e-5 * scale


def test_append_prefill_equals_single_prefill_and_reset_recycles_pages(sb):
    torch = _torch()
    g = SMALL["g2-qknorm"]
    w = si.make_weights(g, seed=24)
    p = si.make_prompts(g.vocab, 2, 40, 50, seed=13)
    sess = make_session(sb, g, w, 16, 2, 8, 256, 128, page_seed=7)
    one = sess.prefill([0, 1], p).cpu().numpy()
    free_after = sb.spiral_kv_free_pages(sess.pool)
    sb.spiral_seq_reset(sess.pool, [0, 1])
    assert sb.spiral_kv_free_pages(sess.pool) == 16 and sb.spiral_seq_len(sess.pool, 0) == 0
    sess.prefill([0, 1], [p[0][:13], p[1][:29]])                 # first turn
    two = sess.prefill([1, 0], [p[1][29:], p[0][13:]]).cpu().numpy()   # next turn appended, other order
    assert sb.spiral_kv_free_pages(sess.pool) == free_after
    assert sb.spiral_seq_len(sess.pool, 0) == len(p[0]) and sb.spiral_seq_len(sess.pool, 1) == len(p[1])
    scale = np.abs(one).max()
    assert np.abs(two[::-1] - one).max() <= 1e-5 * scale
    want = np.stack([od.forward_full(g, w, p[b], logits_at=[len(p[b]) - 1])[0] for b in range(2)])
    assert_logits_close(two[::-1], want, "append prefill")
    sess.close()


def test_games_of_different_lengths_share_the_batch(sb):
    """Self-play shape of the workload: each slot plays games of two turns (history, response, the
    opponent's move appended to the cached history, second response); responses have different
    lengths, so slots finish at different steps, are reset and refilled with the next game while the
    others keep decoding, and every decode call lists only the live slots.  Every logits row the
    library returns is checked against a full recompute of that game's token sequence."""
    torch = _torch()
    rng = np.random.default_rng(31)
    g = SMALL["g4-qknorm"]
    w = si.make_weights(g, seed=26)
    n_slots, n_games = 4, 9
    games = []
    for i in range(n_games):
        games.append({"hist": rng.integers(0, g.vocab, rng.integers(1, 40)), "resp1": rng.integers(0, g.vocab, rng.integers(1, 14)),
                      "move": rng.integers(0, g.vocab, rng.integers(1, 20)), "resp2": rng.integers(0, g.vocab, rng.integers(1, 14))})
    sess = make_session(sb, g, w, n_pages=40, max_seqs=n_slots, max_blocks=8, max_rows=256, max_context=128, page_seed=8)
    free0 = sb.spiral_kv_free_pages(sess.pool)
    # per slot: the game it plays, its phase, and the (position, logits) rows collected for the game
    slot_game = [None] * n_slots
    todo = list(range(n_games))
    got = {i: [] for i in range(n_games)}
    state = {}

    def start(slot):
        gi = todo.pop(0)
        slot_game[slot] = gi
        lg = sess.prefill([slot], [games[gi]["hist"]]).cpu().numpy()[0]
        state[gi] = {"phase": 1, "k": 0, "len": len(games[gi]["hist"])}
        got[gi].append((state[gi]["len"] - 1, lg))

    for slot in range(n_slots):
        start(slot)
    calls = 0
    while any(x is not None for x in slot_game):
        live = [s_ for s_ in range(n_slots) if slot_game[s_] is not None]
        toks = []
        for s_ in live:
            gi = slot_game[s_]; st = state[gi]
            toks.append(games[gi]["resp1" if st["phase"] == 1 else "resp2"][st["k"]])
        order = list(rng.permutation(len(live)))                      # the call may list the live slots in any order
        ids = [live[j] for j in order]
        tin = torch.tensor([int(toks[j]) for j in order], dtype=torch.int32, device=sess.device)
        lg = sess.decode_step(ids, tin, sess.new_logits(len(ids))).cpu().numpy()
        calls += 1
        for row, s_ in enumerate(ids):
            gi = slot_game[s_]; st = state[gi]
            st["len"] += 1; st["k"] += 1
            got[gi].append((st["len"] - 1, lg[row]))
            resp = games[gi]["resp1" if st["phase"] == 1 else "resp2"]
            if st["k"] == len(resp):
                if st["phase"] == 1:                                   # the opponent moved: append to the cached history
                    lgm = sess.prefill([s_], [games[gi]["move"]]).cpu().numpy()[0]
                    st["len"] += len(games[gi]["move"]); st["phase"] = 2; st["k"] = 0
                    got[gi].append((st["len"] - 1, lgm))
                else:                                                  # game over: free the slot, start the next game
                    assert sb.spiral_seq_len(sess.pool, s_) == st["len"]
                    sb.spiral_seq_reset(sess.pool, [s_])
                    slot_game[s_] = None
                    if todo:
                        start(s_)
    assert sb.spiral_kv_free_pages(sess.pool) == free0
    worst = 0.0
    for gi, gm in enumerate(games):
        seq = np.concatenate([gm["hist"], gm["resp1"], gm["move"], gm["resp2"]])
        pos = [p_ for p_, _ in got[gi]]
        want = od.forward_full(g, w, seq, logits_at=pos)
        worst = max(worst, assert_logits_close(np.stack([r for _, r in got[gi]]), want, f"game {gi}"))
    print(f"{n_games} games over {n_slots} slots in {calls} decode calls: max|dlogit|/std = {worst:.3e}")
    sess.close()


@pytest.mark.parametrize("B", [300, 1024])
def test_large_decode_batch_spans_row_tiles_and_upload_chunks(sb, B):
    """300 and 1024 (the most a call takes) sequences in one decode call: more than one 128-row GEMM tile (the
    large-M kernels at 1024), several by-value uploads of ids / page counts, and an attention stream whose
    workgroup ranges each hold many short sequences."""
    g = SMALL["g2-qknorm"]
    w = si.make_weights(g, seed=28)
    steps = 3
    prompts = si.make_prompts(g.vocab, B, 1, 40, seed=17)
    forced = si.make_forced_tokens(g.vocab, B, steps, seed=18)
    n_pages = sum((len(p) + steps + 16) // 16 for p in prompts) + 4
    sess = make_session(sb, g, w, n_pages=n_pages, max_seqs=B, max_blocks=4, max_rows=sum(len(p) for p in prompts),
                        max_context=64, page_seed=10)
    got_logits, got_tok = run_teacher_forced(sb, sess, g, prompts, forced)
    worst = 0.0
    for b in list(range(0, B, 29)) + [127, 128, 129, 255, 256, B - 1]:
        want = oracle_teacher_forced(g, w, prompts[b], forced[:, b])
        worst = max(worst, assert_logits_close(got_logits[:, b], want, f"large batch seq {b}"))
    print(f"B = {B}: max|dlogit|/std = {worst:.3e}")
    sess.close()


def test_errors_leave_state_untouched(sb):
    torch = _torch()
    g = SMALL["g1-mha"]
    w = si.make_weights(g, seed=25)
    sess = make_session(sb, g, w, n_pages=4, max_seqs=3, max_blocks=3, max_rows=128, max_context=64)
    prompts = si.make_prompts(g.vocab, 2, 20, 20, seed=14)
    logits = sess.prefill([0, 1], prompts)                                   # 2 pages each: pool now empty
    ref = logits.cpu().numpy().copy()
    assert sb.spiral_kv_free_pages(sess.pool) == 0
    tok = torch.zeros(3, dtype=torch.int32, device=sess.device)
    lg3 = sess.new_logits(3)
    with pytest.raises(sb.SpiralError) as e:                                 # third sequence needs a page
        sb.spiral_decode_step(sess.model, sess.pool, [0, 1, 2], tok, sess.ws, lg3)
    assert e.value.code == sb.SPIRAL_ERR_OOM_KV
    with pytest.raises(sb.SpiralError) as e:
        sb.spiral_decode_step(sess.model, sess.pool, [0, 0], tok, sess.ws, lg3)
    assert e.value.code == sb.SPIRAL_ERR_INVALID_ARG
    with pytest.raises(sb.SpiralError) as e:
        sb.spiral_decode_step(sess.model, sess.pool, [0, 7], tok, sess.ws, lg3)
    assert e.value.code == sb.SPIRAL_ERR_INVALID_ARG
    with pytest.raises(sb.SpiralError) as e:                                 # would exceed the block table
        sess.prefill([0], [np.zeros(40, dtype=np.int32)])
    assert e.value.code == sb.SPIRAL_ERR_OOM_KV
    small_ws = sess.ws[:1024]
    with pytest.raises(sb.SpiralError) as e:
        sb.spiral_decode_step(sess.model, sess.pool, [0, 1], tok, small_ws, lg3)
    assert e.value.code == sb.SPIRAL_ERR_OOM_KV
    assert [sb.spiral_seq_len(sess.pool, i) for i in range(3)] == [20, 20, 0]
    # the sequences still decode correctly afterwards
    forced = si.make_forced_tokens(g.vocab, 2, 1, seed=15)
    lg2 = sess.new_logits(2)
    sess.decode_step([0, 1], torch.from_numpy(forced[0]).to(sess.device), lg2)
    for b in range(2):
        want = oracle_teacher_forced(g, w, prompts[b], forced[:, b])
        assert_logits_close(np.stack([ref[b], lg2[b].cpu().numpy()]), want, f"after errors seq {b}")
    sess.close()


def test_same_inputs_give_bit_identical_logits(sb):
    g = SMALL["g7-bias"]
    w = si.make_weights(g, seed=26)
    prompts = si.make_prompts(g.vocab, 5, 30, 90, seed=16)
    forced = si.make_forced_tokens(g.vocab, 5, 5, seed=17)
    outs = []
    for _ in range(2):
        sess = make_session(sb, g, w, 64, 5, 8, 512, 128, page_seed=8)
        outs.append(run_teacher_forced(sb, sess, g, prompts, forced)[0])
        sess.close()
    assert np.array_equal(outs[0], outs[1])


# ------------------------------------------------------------------------------------------------
# sampler
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("V", [151936, 1000, 7])
def test_sampler_matches_oracle(sb, V):
    torch = _torch()
    B = 16
    logits = si.make_uniform_noise_free_logits(B, V, seed=30)
    dl = torch.from_numpy(logits).cuda()
    out = torch.empty(B, dtype=torch.int32, device="cuda")
    seq_ids = np.arange(100, 100 + B, dtype=np.int32)
    steps = np.arange(B, dtype=np.int32) * 37
    # greedy
    sb.spiral_sample(dl, B, V, 0.0, 0, None, None, None, out)
    want, margins = osamp.sample(logits, 0.0, 0, seq_ids, steps)
    assert np.array_equal(out.cpu().numpy(), want)                  # exact: no arithmetic involved
    # generated noise, T = 1.0 (the actor setting) and T = 0.6
    for T in (1.0, 0.6):
        sb.spiral_sample(dl, B, V, T, 1234, seq_ids, steps, None, out)
        want, margins = osamp.sample(logits, T, 1234, seq_ids, steps)
        n = assert_tokens_match(out.cpu().numpy(), want, margins, f"sampled V={V} T={T}")
        assert n >= B // 2 or V < 100
    # shared-noise mode: the oracle's noise buffer is handed to the kernel -> identical everywhere
    noise = np.stack([osamp.gumbel_noise(99, int(seq_ids[b]), int(steps[b]), V) for b in range(B)])
    sb.spiral_sample(dl, B, V, 1.0, 0, None, None, torch.from_numpy(noise).cuda(), out)
    want, margins = osamp.sample(logits, 1.0, 0, seq_ids, steps, noise=noise)
    assert np.array_equal(out.cpu().numpy(), want)


def test_sampler_ties_take_lowest_index_and_large_batch(sb):
    torch = _torch()
    V = 5000
    logits = np.zeros((300, V), dtype=np.float32)
    logits[:, 4321] = 2.0
    logits[:, 77] = 2.0
    out = torch.empty(300, dtype=torch.int32, device="cuda")
    sb.spiral_sample(torch.from_numpy(logits).cuda(), 300, V, 0.0, 0, None, None, None, out)
    assert (out.cpu().numpy() == 77).all()


def test_generated_noise_follows_the_specified_stream(sb):
    """With zero logits the sampled token is the argmax of the noise itself."""
    torch = _torch()
    V, B = 4096, 8
    out = torch.empty(B, dtype=torch.int32, device="cuda")
    seq_ids = np.array([0, 1, 2, 3, 1000, 65535, 7, 7], dtype=np.int32)
    steps = np.array([0, 0, 5, 8191, 1, 2, 3, 4], dtype=np.int32)
    sb.spiral_sample(torch.zeros(B, V, device="cuda"), B, V, 1.0, 2 ** 63 + 11, seq_ids, steps, None, out)
    want = [int(np.argmax(osamp.random_bits(2 ** 63 + 11, int(s), int(t), V) >> np.uint32(9))) for s, t in zip(seq_ids, steps)]
    assert out.cpu().numpy().tolist() == want
