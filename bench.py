#!/usr/bin/env python3
"""Decode-throughput benchmark of the self-play generation path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W [--workload C3]

A "step" is one pass of the whole hot path over the batch: spiral_decode_step (embedding, all
layers, LM head) followed by spiral_sample, free-running (each step consumes the tokens the
previous step sampled).  Inputs (random-init weights, uniform-random prompts, shuffled physical
pages) are synthetic, seeded and resident in HBM before the timed region; prefill is outside it.
Prints ONE JSON line: generated tokens/s, plus the roofline of the dominant kernel (split-K paged
decode attention) measured with HIP events, and the CPU oracle timed on the host as a baseline.
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
PMC_TRAFFIC_OVER_ALGORITHMIC = 1.032      # measured ratio for the decode attention kernel (see profiles/)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_session(wl, total_new_tokens, prefill_group_tokens):
    import torch
    from paper_2506_24119_amd import binding as sb
    from paper_2506_24119_amd import inputs as si

    g = wl.geometry
    dev = "cuda:0"
    t0 = time.time()
    if g.n_layers * g.params_per_layer() > 50_000_000:
        w = si.make_weights_torch(g, wl.seed, dev)
    else:
        w = sb.weights_to_device(si.make_weights(g, wl.seed), dev)
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
                      page_order=si.make_page_order(n_pages, wl.seed), device=dev)
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


def run_steps(sess, sb, ids, logits, tokens, first_step, n, temperature, seed, fused=True):
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


def algorithmic_bytes(g, lens_after_append, B):
    """Bytes one decode step must move: weights of all layers + LM head, the whole KV context read
    once per layer, the appended K/V, and the logits written and read back by the sampler."""
    wbytes = 2 if g.weight_dtype == 1 else 4
    weights = (g.n_layers * g.params_per_layer() + g.vocab * g.d_model) * wbytes
    kv_tok = 2 * g.n_kv_heads * g.head_dim * 2                      # K+V bytes per token per layer (16-bit cache)
    kv_read = int(lens_after_append.sum()) * kv_tok * g.n_layers
    kv_write = B * kv_tok * g.n_layers
    logits = 2 * B * g.vocab * 4
    return weights + kv_read + kv_write + logits, kv_read // g.n_layers


MFMA_PEAK_TFLOPS = 2500.0          # dense 16-bit MFMA peak of MI355X


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
    paper's evaluation setting (temperature 0.6, top-p 0.95) on the step's logits."""
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
    us_trunc = timed(lambda: sb.spiral_sample_truncated(logits, B, g.vocab, 0.6, 0, 0.95, 1, ids, steps, None, out_tok, None))
    nbytes = B * g.vocab * 4
    rep["sample_truncated"] = {"setting": "T=0.6, top-p 0.95", "us": us_trunc, "us_untruncated": us_plain,
                               "logits_bytes": nbytes, "GBps": nbytes / us_trunc / 1e3,
                               "note": "6 passes over the row (max, 4 radix digits of probability mass, draw); ALU/LDS-atomic bound"}
    log(f"[bench] sampler: untruncated {us_plain:.0f} us, T=0.6 top-p 0.95 {us_trunc:.0f} us")
    return rep


def cpu_baseline(wl, prompts, weights_dev, n_steps=48):
    """The oracle's KV-cached decoder (fp32 variant) on the host: one sequence of the batch (the
    shortest prompt), prompt consumed untimed, n_steps decode steps timed."""
    from oracle import decoder as od
    from paper_2506_24119_amd import inputs as si
    import torch
    g = wl.geometry
    t0 = time.time()
    w_host = si.weights_to_host_numpy(weights_dev)
    b = int(np.argmin([len(p) for p in prompts]))
    dec = od.CachedDecoder(g, w_host, dtype=np.float32)
    log(f"[bench] oracle weights widened in {time.time() - t0:.1f}s")
    t0 = time.time()
    lg = dec.prefill(prompts[b])
    log(f"[bench] oracle prefill of {len(prompts[b])} tokens: {time.time() - t0:.1f}s")
    tok = int(np.argmax(lg))
    t0 = time.time()
    for _ in range(n_steps):
        lg = dec.step(tok)
        tok = int(np.argmax(lg))
    dt = time.time() - t0
    cores = torch.get_num_threads()
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        pass
    return {"value": n_steps / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"1 of {wl.batch} sequences (prompt {len(prompts[b])} tokens, consumed untimed), "
                      f"{n_steps} KV-cached decode steps, numpy fp32"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--prefill-group-tokens", type=int, default=16384)
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
    K = args.steps if args.steps is not None else wl.decode_steps
    W = args.warmup
    B = wl.batch
    sess, prompts, lens0 = build_session(wl, W + K, args.prefill_group_tokens)
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
    tokens0 = tokens.clone()

    # ---- warm-up, then the timed region
    run_steps(sess, sb, ids, logits, tokens, 1, W, wl.temperature, seed)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(sess, sb, ids, logits, tokens, 1 + W, K, wl.temperature, seed)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    tok_per_s = B * K / dt
    log(f"[bench] {K} steps in {dt:.3f}s -> {tok_per_s:.0f} tokens/s")

    total_bytes, attn_bytes = 0, 0
    for k in range(K):
        tb, ab = algorithmic_bytes(g, lens0 + W + k + 1, B)
        total_bytes += tb
        attn_bytes += ab * g.n_layers
    step_gbps = total_bytes / dt / 1e9

    # ---- dominant kernel: rewind to the start of the timed region and replay it with HIP events
    roofline = {"bound": "hbm", "kernel": "attn_stream_kernel (paged decode attention, balanced page stream)", "achieved": None,
                "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": None, "traffic": None}
    if not args.no_kernel_timing:
        sb.spiral_seq_truncate(sess.pool, ids, lens0)
        tokens.copy_(tokens0)
        run_steps(sess, sb, ids, logits, tokens, 1, W, wl.temperature, seed)
        torch.cuda.synchronize()
        sb.spiral_profile_begin(sess.model, sb.KERNEL_CLASSES.index("attn_decode"), K * g.n_layers)
        run_steps(sess, sb, ids, logits, tokens, 1 + W, K, wl.temperature, seed)
        ms, n = sb.spiral_profile_end(sess.model)
        assert n == K * g.n_layers, (n, K * g.n_layers)
        achieved = attn_bytes / (ms * 1e-3) / 1e9
        # HBM bytes per launch from rocprofv3 PMC (profiles/attn_decode_c3_pmc_traffic.md): FETCH_SIZE x 2.00
        # (calibrated on plain copies) + WRITE_SIZE x 1.00 = 1.032 x the algorithmic bytes
        roofline.update({"traffic": PMC_TRAFFIC_OVER_ALGORITHMIC * attn_bytes / n,
                         "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on C3, copy-calibrated: "
                                           "1.032 x algorithmic bytes (profiles/attn_decode_c3_pmc_traffic.md)",
                         "achieved": achieved, "frac": achieved / HBM_PEAK_GBPS,
                         "avg_launch_us": 1e3 * ms / n, "launches": n,
                         "algorithmic_bytes_per_launch": attn_bytes / n})
        log(f"[bench] attention: {n} launches, avg {1e3 * ms / n:.1f} us, {achieved:.0f} GB/s")

    out = {
        "metric": "generated tokens/sec on 1 MI355X (Qwen3-4B-shaped decode); % HBM roofline",
        "value": tok_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": 1e3 * dt / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 (bf16 weights widened in registers; f16 activations and KV cache; f32 accumulate)"
                 if "f16 MFMA" in sb.spiral_version() else "bf16",
        "data": "synthetic",
        "config": {"workload": f"{wl.key}: {g.name}-shaped random init, batch {B}, prompts U[{wl.prompt_lo},{wl.prompt_hi}], "
                               f"{K} decode steps, T={wl.temperature} seeded Gumbel-max sampling, 16-token pages",
                   "context_tokens_start": int((lens0 + W).sum()), "context_tokens_end": int((lens0 + W + K).sum())},
        "hbm_step": {"algorithmic_GB_per_step": total_bytes / K / 1e9, "achieved_GBps": step_gbps,
                     "frac_of_8TBps": step_gbps / HBM_PEAK_GBPS},
        "prefill_s": prefill_s,
        "roofline": roofline,
    }
    out["prefill"] = prefill_report(g, prompts, prefill_s, score=False)
    if not args.no_extras and g.weight_dtype == 1 and g.d_model % 128 == 0:
        out["next_rows"] = next_rows(sess, sb, wl, prompts, ids, logits, args.prefill_group_tokens)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, prompts, sess.weights)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
