#!/usr/bin/env python3
"""Decode-throughput benchmark of the self-play generation path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W [--workload C3] [--repeats 3]

A "step" is one pass of the whole hot path over the batch: one spiral_decode_sample_step (embedding, all
layers, LM head feeding the Gumbel-max sampler), free-running (each step consumes the tokens the previous
step sampled).  Inputs (random-init weights, uniform-random prompts, shuffled physical pages) are synthetic,
seeded and resident in HBM before the timed region; prefill is outside it.

Timed region: the workload is the configuration's whole decode run (C3: 512 steps).  When K is smaller than
that, the K timed steps are the window in the middle of the run (steps [P, P + K), P = (run - K) // 2, reached
by untimed steps), so that the context lengths are the run's mean ones rather than its shortest; K equal to
the run length times all of it.  The window is timed `--repeats` times (state rewound with
spiral_seq_truncate, W untimed warm-up steps before each) and the median is reported.

Prints ONE JSON line: generated tokens/s; `roofline` for the dominant kernel (paged decode attention, HIP
events around every launch) plus the whole step's fraction of peak HBM bandwidth and of a streaming read
measured in the same run; `cpu_baseline`, the oracle timed on the host.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0          # dense 16-bit MFMA peak of MI355X
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "attn_decode_c3_pmc_traffic.json")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_session(wl, total_new_tokens, prefill_group_tokens, tune=None, weight_std=0.02):
    import torch
    from paper_2506_24119_amd import binding as sb
    from paper_2506_24119_amd import inputs as si

    g = wl.geometry
    dev = "cuda:0"
    t0 = time.time()
    if g.n_layers * g.params_per_layer() > 50_000_000:
        w = si.make_weights_torch(g, wl.seed, dev, std=weight_std)
    else:
        w = sb.weights_to_device(si.make_weights(g, wl.seed, std=weight_std), dev)
    torch.cuda.synchronize()
    log(f"[bench] weights ready in {time.time() - t0:.1f}s")
    prompts = si.make_prompts(g.vocab, wl.batch, wl.prompt_lo, wl.prompt_hi, wl.seed)
    lens = np.array([len(p) for p in prompts])
    final = lens + total_new_tokens + 1
    blocks = (final + 15) // 16
    n_pages = int(blocks.sum()) + 8
    max_blocks = int(blocks.max())
    max_rows = max(wl.batch, min(int(lens.sum()), prefill_group_tokens + int(lens.max())))
    sess = sb.Session(g, w, n_pages, wl.batch, max_blocks, max_rows, int(final.max()),
                      page_order=si.make_page_order(n_pages, wl.seed), device=dev, tune=tune)
    return sess, prompts, lens


def prefill_all(sess, prompts, group_tokens):
    """Prefill in groups of sequences of at most ~group_tokens tokens; returns logits [B, V]."""
    import torch
    B = len(prompts)
    logits = sess.new_logits(B)
    i = 0
    while i < B:
        j, tok = i, 0
        while j < B and (j == i or tok + len(prompts[j]) <= group_tokens):
            tok += len(prompts[j])
            j += 1
        sess.prefill(np.arange(i, j, dtype=np.int32), prompts[i:j], logits=logits[i:j])
        i = j
    torch.cuda.synchronize()
    return logits


def run_steps(sess, ids, logits, tokens, first_step, n, temperature, seed, fused):
    """n free-running steps: decode the current tokens, sample the next ones.  fused: one call per step
    (spiral_decode_sample_step: the LM head feeds the sampler, no logits are written); otherwise
    spiral_decode_step + spiral_sample through the [B, vocab] logits."""
    B = len(ids)
    step_arr = np.empty(B, dtype=np.int32)
    for k in range(n):
        step_arr.fill(first_step + k)
        if fused:
            sess.decode_sample_step(ids, tokens, temperature, seed, step_arr, tokens)
        else:
            sess.decode_step(ids, tokens, logits)
            sess.sample(logits, temperature, seed, ids, step_arr, tokens)


def algorithmic_bytes(g, lens_after_append, B, fused):
    """Bytes one decode step must move: weights of all layers + LM head, the whole KV context read once per
    layer, the appended K/V, and - only when the sampler is a separate call - the logits written and read back."""
    wbytes = 2 if g.weight_dtype == 1 else 4
    weights = (g.n_layers * g.params_per_layer() + g.vocab * g.d_model) * wbytes
    kv_tok = 2 * g.n_kv_heads * g.head_dim * 2                      # K+V bytes per token per layer (16-bit cache)
    kv_read = int(lens_after_append.sum()) * kv_tok * g.n_layers
    kv_write = B * kv_tok * g.n_layers
    logits = 0 if fused else 2 * B * g.vocab * 4
    return weights + kv_read + kv_write + logits, kv_read // g.n_layers


def prefill_report(g, prompts, seconds, score):
    """Throughput of a packed causal forward over the prompts against the MFMA peak.  flops = 2 x matmul
    parameters per token (+ the LM head on every row when scoring, on one row per sequence otherwise)
    + 4 x hd x Hq per (token, visible token, layer) of attention."""
    lens = np.array([len(p) for p in prompts], dtype=np.float64)
    tokens = float(lens.sum())
    flops = 2.0 * g.n_layers * g.params_per_layer() * tokens
    flops += 4.0 * g.head_dim * g.n_q_heads * g.n_layers * float((lens * (lens + 1) / 2).sum())
    flops += 2.0 * g.vocab * g.d_model * (tokens if score else len(prompts))
    return {"tokens": int(tokens), "seconds": seconds, "tokens_per_s": tokens / seconds, "tflops": flops / seconds / 1e12,
            "frac_of_mfma_peak": flops / seconds / 1e12 / MFMA_PEAK_TFLOPS}


def next_rows(sess, sb, wl, prompts, ids, logits, group_tokens):
    """Measurements of the rows built beyond the decode step: the learner-side scoring pass over the same
    ragged histories (per-token log-probabilities, logits never written) and the truncated sampler in the
    paper's evaluation setting (temperature 0.6, top-p 0.95) on one step's logits."""
    import torch
    g = wl.geometry
    B = len(prompts)
    sb.spiral_seq_reset(sess.pool, ids)
    groups, i = [], 0
    while i < B:
        j, tok = i, 0
        while j < B and (j == i or tok + len(prompts[j]) <= group_tokens):
            tok += len(prompts[j]); j += 1
        toks = torch.from_numpy(np.concatenate(prompts[i:j]).astype(np.int32)).to(sess.device)
        tg = torch.from_numpy(np.concatenate([np.concatenate([p[1:], [-1]]) for p in prompts[i:j]]).astype(np.int32)).to(sess.device)
        groups.append((np.arange(i, j, dtype=np.int32), [len(p) for p in prompts[i:j]], toks, tg,
                       torch.empty(toks.numel(), dtype=torch.float32, device=sess.device)))
        i = j
    def score_all():
        for gi, ln, toks, tg, out in groups:
            sb.spiral_score(sess.model, sess.pool, gi, ln, toks, tg, sess.ws, out)
        torch.cuda.synchronize()
    score_all()
    sb.spiral_seq_reset(sess.pool, ids)
    t0 = time.time()
    score_all()
    score_s = time.time() - t0
    rep = {"score": prefill_report(g, prompts, score_s, score=True)}
    log(f"[bench] scoring pass over {rep['score']['tokens']} tokens: {score_s:.2f}s, {rep['score']['tflops']:.0f} TFLOP/s")

    out_tok = torch.empty(B, dtype=torch.int32, device=sess.device)
    steps = np.zeros(B, dtype=np.int32)
    def timed(fn, n=20):
        fn(); torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n * 1e3
    us_plain = timed(lambda: sb.spiral_sample(logits, B, g.vocab, 1.0, 1, ids, steps, None, out_tok))
    us_single = timed(lambda: sb.spiral_sample_truncated(logits, B, g.vocab, 0.6, 0, 0.95, 1, ids, steps, None, out_tok, None))
    need = sb.spiral_sample_truncated_workspace_bytes(B, g.vocab)
    work = torch.empty(need, dtype=torch.uint8, device=sess.device)
    us_trunc = timed(lambda: sb.spiral_sample_truncated_ws(logits, B, g.vocab, 0.6, 0, 0.95, 1, ids, steps, None, out_tok, None,
                                                           work, need))
    nbytes = B * g.vocab * 4
    rep["sample_truncated"] = {"setting": "T=0.6, top-p 0.95", "call": "spiral_sample_truncated_ws", "us": us_trunc,
                               "sweeps_of_the_logits": 3, "us_single_kernel": us_single, "us_untruncated": us_plain,
                               "workspace_bytes": need, "logits_bytes": nbytes, "GBps": 3 * nbytes / us_trunc / 1e3}
    log(f"[bench] sampler: untruncated {us_plain:.0f} us, T=0.6 top-p 0.95 {us_trunc:.0f} us on a workspace, "
        f"{us_single:.0f} us in the single kernel")
    return rep


def host_cpu():
    """(model name, physical cores) of this machine, from /proc/cpuinfo."""
    model, cores = "unknown", set()
    try:
        phys = core = None
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name") and model == "unknown":
                model = line.split(":", 1)[1].strip()
            elif line.startswith("physical id"):
                phys = line.split(":", 1)[1].strip()
            elif line.startswith("core id"):
                core = line.split(":", 1)[1].strip()
            elif not line.strip():
                if phys is not None and core is not None:
                    cores.add((phys, core))
                phys = core = None
    except OSError:
        pass
    return model, (len(cores) or (os.cpu_count() or 1))


def cpu_baseline(wl, prompts, weights_dev, n_seqs=4, n_steps=16):
    """The oracle's KV-cached decoder (its fp32 variant, to bound the sample) on the host: sequences 0..n_seqs-1
    of the batch one after the other, each prompt consumed untimed, then n_steps greedy decode steps timed."""
    from oracle import decoder as od
    from paper_2506_24119_amd import inputs as si
    import torch
    g = wl.geometry
    t0 = time.time()
    w_host = si.weights_to_host_numpy(weights_dev)
    dec = od.CachedDecoder(g, w_host, dtype=np.float32)
    log(f"[bench] oracle weights widened in {time.time() - t0:.1f}s")
    n_seqs = min(n_seqs, len(prompts))
    timed_s, timed_tokens = 0.0, 0
    for b in range(n_seqs):
        dec.k = [np.zeros((0, g.n_kv_heads, g.head_dim), np.float32) for _ in dec.layers]       # a fresh, empty cache
        dec.v = [np.zeros((0, g.n_kv_heads, g.head_dim), np.float32) for _ in dec.layers]
        dec.n = 0
        t0 = time.time()
        lg = dec.prefill(prompts[b])
        log(f"[bench] oracle sequence {b}: prefill of {len(prompts[b])} tokens {time.time() - t0:.1f}s")
        tok = int(np.argmax(lg))
        t0 = time.time()
        for _ in range(n_steps):
            lg = dec.step(tok)
            tok = int(np.argmax(lg))
        timed_s += time.time() - t0
        timed_tokens += n_steps
    threads = torch.get_num_threads()
    try:
        from threadpoolctl import threadpool_info
        threads = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        pass
    model, phys = host_cpu()
    rate = timed_tokens / timed_s
    return {"value": rate, "unit": "tokens/s", "cores": int(threads), "kind": "oracle", "cpu_model": model, "physical_cores": phys,
            "sample": f"sequences 0..{n_seqs - 1} of {wl.batch} one after the other (prompts of "
                      f"{[len(p) for p in prompts[:n_seqs]]} tokens consumed untimed), {n_steps} KV-cached decode steps each timed, "
                      f"numpy fp32 on {threads} threads",
            "extrapolated_full_batch_tokens_per_s": rate,
            "extrapolation_note": "the oracle decodes one sequence at a time, so its rate for the whole batch is the same "
                                  "tokens/s (the batch takes batch/n_seqs times as long), not a sum over sequences"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--repeats", type=int, default=3)
    ap.add_argument("--window", default="centered", choices=["centered", "start"],
                    help="where K < run-length timed steps sit in the decode run")
    ap.add_argument("--unfused", action="store_true", help="spiral_decode_step + spiral_sample instead of the fused step")
    ap.add_argument("--tune", default=None, help="spiral_model_tune spec (launch decompositions; measurement only)")
    ap.add_argument("--prefill-group-tokens", type=int, default=16384)
    ap.add_argument("--weight-std", type=float, default=0.02,
                    help="standard deviation of the random-init matrices (the recipe's is 0.02).  0 makes every operand "
                         "zero: a diagnostic of how far the matrix cores' power limit, which depends on the operand "
                         "bits, sets the large-M GEMM times; its line is marked and is not a result")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the scoring-pass and truncated-sampler measurements")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy kernel (reference dispatch for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU (one process, one MI355X); run with --gpus 1. "
                 "Sequences are independent, so N GPUs would each run this same loop on 1/N of the batch.")

    import torch
    from paper_2506_24119_amd import binding as sb
    from paper_2506_24119_amd import inputs as si
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    log("[bench]", sb.spiral_version())

    if args.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                    # 1 GiB read + 1 GiB written by one elementwise copy kernel
        torch.cuda.synchronize()
        del src, dst

    wl = si.WORKLOADS[args.workload]
    g = wl.geometry
    run_len = wl.decode_steps
    K = args.steps if args.steps is not None else run_len
    W = args.warmup
    R = max(1, args.repeats)
    B = wl.batch
    fused = (not args.unfused) and g.weight_dtype == 1 and g.d_model % 128 == 0 and g.vocab % 16 == 0
    # the timed window [P, P + K) of the run; the W warm-up steps are the ones just before it
    P = max(W, (run_len - K) // 2) if (args.window == "centered" and K < run_len) else W
    sess, prompts, lens0 = build_session(wl, P + K, args.prefill_group_tokens, tune=args.tune, weight_std=args.weight_std)
    ids = np.arange(B, dtype=np.int32)
    seed = 1000 + wl.seed

    prefill_all(sess, prompts, args.prefill_group_tokens)              # untimed first pass (code objects, caches)
    sb.spiral_seq_reset(sess.pool, ids)
    t0 = time.time()
    logits = prefill_all(sess, prompts, args.prefill_group_tokens)
    prefill_s = time.time() - t0
    log(f"[bench] prefill of {int(lens0.sum())} tokens: {prefill_s:.2f}s")
    tokens = torch.empty(B, dtype=torch.int32, device=sess.device)
    sess.sample(logits, wl.temperature, seed, ids, np.zeros(B, dtype=np.int32), tokens)

    # ---- untimed steps up to the warm-up point of the window; the state there is what every repeat starts from
    run_steps(sess, ids, logits, tokens, 1, P - W, wl.temperature, seed, fused)
    torch.cuda.synchronize()
    lens_start = (lens0 + (P - W)).astype(np.int32)
    tokens_start = tokens.clone()

    def rewind():
        sb.spiral_seq_truncate(sess.pool, ids, lens_start)
        tokens.copy_(tokens_start)

    times = []
    for r in range(R):
        rewind()
        run_steps(sess, ids, logits, tokens, 1 + P - W, W, wl.temperature, seed, fused)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(sess, ids, logits, tokens, 1 + P, K, wl.temperature, seed, fused)
        torch.cuda.synchronize()
        times.append(time.perf_counter() - t0)
        log(f"[bench] repeat {r}: {K} steps in {times[-1]:.3f}s -> {B * K / times[-1]:.0f} tokens/s")
    dt = float(np.median(times))
    tok_per_s = B * K / dt

    total_bytes, attn_bytes = 0, 0
    for k in range(K):
        tb, ab = algorithmic_bytes(g, lens0 + P + k + 1, B, fused)
        total_bytes += tb
        attn_bytes += ab * g.n_layers
    step_gbps = total_bytes / dt / 1e9

    # ---- what this GPU streams: a pure load kernel over a buffer the size of one attention launch's K/V
    probe_bytes = int(min(max(attn_bytes // max(K * g.n_layers, 1), 64 << 20), sess.pool_mem.numel()) // 4096 * 4096)
    stream_gbps = sb.spiral_probe_stream_read(sess.pool_mem, probe_bytes, iters=10)
    log(f"[bench] streaming read of {probe_bytes / 1e6:.0f} MB: {stream_gbps:.0f} GB/s")

    # ---- dominant kernel: replay the window with HIP events around every decode-attention launch
    roofline = {"bound": "hbm", "kernel": "attn_stream_kernel (paged decode attention, balanced page stream)", "achieved": None,
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": None, "traffic": None}
    if not args.no_kernel_timing:
        rewind()
        run_steps(sess, ids, logits, tokens, 1 + P - W, W, wl.temperature, seed, fused)
        torch.cuda.synchronize()
        sb.spiral_profile_begin(sess.model, sb.KERNEL_CLASSES.index("attn_decode"), K * g.n_layers)
        run_steps(sess, ids, logits, tokens, 1 + P, K, wl.temperature, seed, fused)
        ms, n = sb.spiral_profile_end(sess.model)
        assert n == K * g.n_layers, (n, K * g.n_layers)
        achieved = attn_bytes / (ms * 1e-3) / 1e9
        roofline.update({"achieved": achieved, "frac": achieved / HBM_PEAK_GBPS, "avg_launch_us": 1e3 * ms / n, "launches": n,
                         "algorithmic_bytes_per_launch": attn_bytes / n,
                         "frac_of_measured_stream": achieved / stream_gbps})
        try:
            tj = json.load(open(TRAFFIC_JSON))
            roofline["traffic"] = tj["hbm_bytes_over_algorithmic_bytes"] * attn_bytes / n
            roofline["traffic_source"] = {k: tj[k] for k in ("hbm_bytes_over_algorithmic_bytes", "measured_at_commit", "method", "file")}
        except (OSError, KeyError, ValueError) as e:
            roofline["traffic_source"] = f"unavailable: {e}"
        log(f"[bench] attention: {n} launches, avg {1e3 * ms / n:.1f} us, {achieved:.0f} GB/s")
    # the quantity the target is stated on: algorithmic bytes of the whole step / step time
    roofline.update({"step_achieved": step_gbps, "step_frac": step_gbps / HBM_PEAK_GBPS,
                     "step_frac_of_measured_stream": step_gbps / stream_gbps, "measured_stream_GBps": stream_gbps,
                     "step_algorithmic_GB": total_bytes / K / 1e9})

    window = "whole run" if K >= run_len else f"steps [{P}, {P + K}) of the {run_len}-step run ({args.window} window)"
    out = {
        "metric": "generated tokens/sec on 1 MI355X (Qwen3-4B-shaped decode); % HBM roofline",
        "value": tok_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": 1e3 * dt / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 (bf16 weights widened in registers; f16 activations and KV cache; f32 accumulate)"
                 if "f16 MFMA" in sb.spiral_version() else "bf16",
        "data": "synthetic" if args.weight_std == 0.02 else f"synthetic, DIAGNOSTIC weight std {args.weight_std} (not the workload's recipe)",
        "config": {"workload": f"{wl.key}: {g.name}-shaped random init, batch {B}, prompts U[{wl.prompt_lo},{wl.prompt_hi}], "
                               f"{run_len} decode steps, T={wl.temperature} seeded Gumbel-max sampling, 16-token pages; timed: {window}",
                   "timed_window": [P, P + K], "run_steps": run_len, "repeats": R, "repeat_seconds": times,
                   "step_call": "spiral_decode_sample_step" if fused else "spiral_decode_step + spiral_sample",
                   "context_tokens_start": int((lens0 + P).sum()), "context_tokens_end": int((lens0 + P + K).sum())},
        "hbm_step": {"algorithmic_GB_per_step": total_bytes / K / 1e9, "achieved_GBps": step_gbps,
                     "frac_of_8TBps": step_gbps / HBM_PEAK_GBPS},
        "prefill_s": prefill_s,
        "roofline": roofline,
    }
    out["prefill"] = prefill_report(g, prompts, prefill_s, score=False)
    if not args.no_extras and g.weight_dtype == 1 and g.d_model % 128 == 0:
        sess.decode_step(ids, tokens, logits)          # one step's logits for the sampler timings
        out["next_rows"] = next_rows(sess, sb, wl, prompts, ids, logits, args.prefill_group_tokens)
    out["saturated_activation_stores"] = sess.saturation_count()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, prompts, sess.weights)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
