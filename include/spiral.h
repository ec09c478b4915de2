/*
 * spiral.h — C ABI of the MI355X (gfx950) self-play decode library.
 *
 * The library implements the computation that dominates SPIRAL's run time: the
 * batched autoregressive generation y ~ pi_theta(. | s) of every game turn
 * (Sec. 3 "Self-play"; Alg. 1, generation step) with the actor's sampling
 * settings (hyper-parameter table, App. D: temperature 1.0, top-p 1.0, top-k -1,
 * i.e. an untruncated categorical), plus the role-conditioned advantage
 * estimation baseline (Sec. 3, RAE equation; Alg. 1, policy-optimisation loop).
 *
 * General rules
 *  - Every function returns SPIRAL_OK (0) or a negative SPIRAL_ERR_* code; it
 *    never throws and never aborts.  spiral_last_error() returns a thread-local
 *    description of the last failure on the calling thread.
 *  - "dev" pointers are HIP device pointers, "host" pointers are ordinary host
 *    memory.  The caller owns ALL device memory (weights, KV pool, workspace,
 *    logits, token buffers) and the stream.  The library never allocates or
 *    frees device memory and never synchronises the stream; all device work is
 *    enqueued on the stream that is passed in (`stream` is a hipStream_t, NULL =
 *    the default stream).  Host arrays are consumed before the call returns.
 *  - Opaque host objects (model, pool, RAE state) are created and freed by the
 *    library.  Calls on the same object must not overlap.
 *  - A failed call leaves sequence lengths and page tables unchanged: the sequences' lengths, their page lists
 *    and the free list are host-side state that is advanced only after every launch of the call was accepted
 *    (pages taken earlier in the call are returned).  After SPIRAL_ERR_HIP some kernels of the call may already
 *    be enqueued; they write only beyond the sequences' recorded lengths and into the workspace.
 *  - Precision: 16-bit weights are bf16 as given; activations, q, the cached K/V and the softmax weights are IEEE
 *    half, all sums are fp32.  A value outside half's range (|x| > 65504) is stored as +-65504 and a NaN stays a
 *    NaN; every such store increments a counter in the KV pool (spiral_kv_pool_status_offset) so that a caller
 *    running a checkpoint with large activations can detect it.
 */
#ifndef SPIRAL_H
#define SPIRAL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPIRAL_OK               0
#define SPIRAL_ERR_INVALID_ARG (-1)  /* null pointer, bad id, duplicate sequence, misaligned buffer */
#define SPIRAL_ERR_SHAPE       (-2)  /* geometry or size the kernels do not support */
#define SPIRAL_ERR_OOM_KV      (-3)  /* not enough free KV pages / block-table slots / workspace */
#define SPIRAL_ERR_NOT_LOADED  (-4)  /* object handle is null or already freed */
#define SPIRAL_ERR_HIP         (-5)  /* a HIP runtime call failed (text in spiral_last_error) */

#define SPIRAL_WEIGHT_FP32 0
#define SPIRAL_WEIGHT_BF16 1

#define SPIRAL_MAX_BATCH 1024        /* sequences per prefill / decode / sample call */

/* Decoder geometry.  The paper names its policies only by model family (Sec. 4,
 * "Models"); the block is the standard pre-norm decoder of those families:
 * RMSNorm -> QKV (+bias | per-head q/k RMSNorm) -> RoPE (rotate-half) -> causal
 * GQA attention -> output projection + residual -> RMSNorm -> SwiGLU MLP +
 * residual; final RMSNorm and LM head. */
typedef struct spiral_model_config {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab;
    float   rope_theta;      /* RoPE base; pair (j, j+head_dim/2) turns by pos * theta^(-2j/head_dim) */
    float   rms_eps;         /* added to the mean square inside the square root */
    int32_t qk_norm;         /* 1: RMSNorm over head_dim of every q and k head (gain shared by heads), before RoPE */
    int32_t qkv_bias;        /* 1: bias on the q, k, v projections, added before RoPE */
    int32_t tie_lm_head;     /* informational: lm_head pointer aliases the embedding */
    int32_t weight_dtype;    /* SPIRAL_WEIGHT_FP32 or SPIRAL_WEIGHT_BF16 (matrices, embedding, biases) */
    int32_t kv_block_tokens; /* tokens per KV page; must be 16 */
} spiral_model_config;

/* Order of the device weight pointer table handed to spiral_model_load:
 *   [0] embedding [vocab, d_model]   [1] final RMSNorm gain [d_model] (fp32)   [2] lm_head [vocab, d_model]
 *   then, for layer l, 14 slots starting at 3 + 14*l, in the order below.  Matrices are row-major
 *   [out_features, in_features] in weight_dtype; biases in weight_dtype; all gains are fp32.
 *   Slots a geometry does not use (biases, q/k norms) are NULL. */
enum spiral_layer_slot {
    SPIRAL_W_ATTN_NORM = 0, /* [d_model] fp32 */
    SPIRAL_W_Q, SPIRAL_W_K, SPIRAL_W_V,      /* [Hq*hd, d], [Hkv*hd, d], [Hkv*hd, d] */
    SPIRAL_W_BQ, SPIRAL_W_BK, SPIRAL_W_BV,   /* [Hq*hd], [Hkv*hd], [Hkv*hd] or NULL */
    SPIRAL_W_Q_NORM, SPIRAL_W_K_NORM,        /* [hd] fp32 or NULL */
    SPIRAL_W_O,                              /* [d, Hq*hd] */
    SPIRAL_W_MLP_NORM,                       /* [d_model] fp32 */
    SPIRAL_W_GATE, SPIRAL_W_UP,              /* [ffn, d] */
    SPIRAL_W_DOWN,                           /* [d, ffn] */
    SPIRAL_LAYER_SLOTS                       /* = 14 */
};

typedef struct spiral_model   spiral_model;
typedef struct spiral_kv_pool spiral_kv_pool;
typedef struct spiral_rae     spiral_rae;

const char* spiral_last_error(void);
const char* spiral_version(void);

/* ---- model ------------------------------------------------------------------------------------
 * Records the geometry and the caller's device weight pointers (no copy, no repack; the weights
 * must stay valid and unchanged while the model is in use).  host_dev_weights: host array of
 * n_weights = 3 + 14*n_layers device pointers in the order above, every matrix 16-byte aligned.
 * Errors: INVALID_ARG (null / missing required pointer / misaligned / wrong n_weights),
 * SHAPE (head_dim not in {32,64,128}; Hq not a multiple of Hkv or Hq/Hkv > 16; kv_block_tokens != 16;
 * for bf16 weights: d_model, Hq*hd, ffn_dim not multiples of 32, or any projection width not a
 * multiple of 16). */
int  spiral_model_load(const spiral_model_config* cfg, const void* const* host_dev_weights,
                       int n_weights, spiral_model** out);
void spiral_model_free(spiral_model* m);

/* Optional: copy the projection matrices and the LM head into the order the matrix-core operands are
 * loaded in (1 KB blocks of 32 rows x 16 k; gate and up rows interleaved), so that every wave load
 * reads whole cache lines.  dev_buffer: caller-owned device memory of at least
 * spiral_model_repack_bytes(m) bytes (0: this geometry cannot be repacked), 256-byte aligned, which
 * must stay valid as long as the model; the original weights must stay valid too (embedding rows,
 * norms and biases are read from them).  The copies are enqueued on `stream`; calls that follow on the
 * same stream use them.  Same results bit for bit.  Errors: NOT_LOADED, SHAPE, INVALID_ARG, HIP. */
size_t spiral_model_repack_bytes(const spiral_model* m);
int spiral_model_repack(spiral_model* m, void* dev_buffer, size_t bytes, void* stream);

/* Measurement / test hook: overrides the launch decomposition the library would choose from the geometry.
 * spec is a comma-separated list of key=value items (unknown keys are ignored): "qkv=R:S", "o=R:S", "down=R:S"
 * (weight rows per workgroup : K splits of that projection), "gu=R", "lm=R", "chunk=P" (least pages per
 * decode-attention workgroup), "wgs=N" (workgroups of the decode attention), "frag=0|1" (use the repacked weights),
 * "fuse_qkv=0|1" (large row counts: q/k/v post-processing inside the projection kernel or as its own kernel),
 * "fail_after=N" (error-path tests: the N-th
 * kernel launch of the layer stack from now on is not made and reports a launch failure).  Results stay within
 * the parity tolerance for every setting; the defaults are the measured best.  "frag" must be set before
 * spiral_model_repack, the others at any time between calls.  Errors: NOT_LOADED, INVALID_ARG. */
int spiral_model_tune(spiral_model* m, const char* spec);

/* Bytes of device workspace a prefill over at most max_rows packed prompt tokens, or a decode step
 * over at most max_rows sequences whose context is at most max_context tokens, needs.
 * Returns 0 on bad arguments. */
size_t spiral_workspace_bytes(const spiral_model* m, int max_rows, int max_context);

/* ---- paged KV cache ---------------------------------------------------------------------------
 * One pool holds the K and V of every layer for up to max_seqs sequences in n_pages pages of 16
 * tokens; a sequence owns at most max_blocks_per_seq pages.  Layout inside dev_mem (all managed by
 * the library): block table int32 [max_seqs, max_blocks_per_seq], a 256-byte status block, then the
 * pages, 16-bit (IEEE half): [layer][page][kv_head]{ K (16 tokens x head_dim), V (head_dim x 16 tokens) },
 * each stored in the element order of the matrix-core operands (an internal layout).  Sequence lengths are
 * host-side state of the pool object.
 * spiral_kv_pool_bytes gives the size dev_mem must have (0 on bad arguments); dev_mem must be
 * 256-byte aligned.  host_page_order (n_pages distinct ids in [0,n_pages), or NULL for ascending)
 * is the order in which free pages are handed out.  Creation enqueues a zero fill of the pool on
 * `stream`.  Sequence ids are the integers [0, max_seqs); all start empty. */
size_t spiral_kv_pool_bytes(const spiral_model* m, int n_pages, int max_seqs, int max_blocks_per_seq);
int    spiral_kv_pool_create(const spiral_model* m, void* dev_mem, size_t bytes, int n_pages,
                             int max_seqs, int max_blocks_per_seq, const int32_t* host_page_order,
                             void* stream, spiral_kv_pool** out);
void   spiral_kv_pool_free(spiral_kv_pool* p);
/* Byte offset inside dev_mem of the pool's status block: int32 [0] counts the activation values that did not
 * fit the 16-bit format since the pool was created (see "Precision" above; 0 in a healthy run).  The caller
 * reads it with a copy of its own, after synchronising the stream.  Negative error code on a null pool. */
long long spiral_kv_pool_status_offset(const spiral_kv_pool* p);
/* Empties the listed sequences and returns their pages to the free list (in reverse order of use).  Host-side
 * bookkeeping only: nothing is enqueued (`stream` is accepted for symmetry and ignored). */
int    spiral_seq_reset(spiral_kv_pool* p, const int32_t* host_seq_ids, int n, void* stream);
/* Shortens the listed sequences to host_new_lens[i] tokens (0 <= new length <= current length) and
 * returns the pages that are no longer needed; the cached K/V of the kept prefix stay valid.  Used
 * to drop a discarded generation and continue from the kept history (e.g. replaying a turn).
 * Errors: INVALID_ARG (bad id, duplicate, length out of range); nothing is modified then. */
int    spiral_seq_truncate(spiral_kv_pool* p, const int32_t* host_seq_ids, const int32_t* host_new_lens,
                           int n, void* stream);
/* Host-side view: tokens cached for a sequence (negative error code on a bad id); free pages. */
int    spiral_seq_len(const spiral_kv_pool* p, int seq_id);
int    spiral_kv_free_pages(const spiral_kv_pool* p);

/* ---- prefill ----------------------------------------------------------------------------------
 * Appends host_lens[i] >= 1 tokens to sequence host_seq_ids[i] (i < B; ids distinct) and returns the
 * next-token logits after each sequence's last appended token.  A sequence may already hold a
 * history (a new game turn appended to earlier turns): positions continue from its current length.
 * dev_tokens_packed: int32 [sum(host_lens)], the sequences' tokens back to back, ids in [0, vocab).
 * dev_logits: fp32 [B, vocab].  dev_ws/ws_bytes: workspace of at least
 * spiral_workspace_bytes(m, sum(host_lens), longest resulting context), 256-byte aligned.
 * Errors: INVALID_ARG, OOM_KV (pages, block-table slots or workspace too small), HIP. */
int spiral_prefill(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids,
                   const int32_t* host_lens, int B, const int32_t* dev_tokens_packed,
                   void* dev_ws, size_t ws_bytes, float* dev_logits, void* stream);

/* ---- decode step ------------------------------------------------------------------------------
 * One autoregressive step for B distinct, non-empty sequences: sequence host_seq_ids[i] consumes
 * token dev_in_tokens[i] at position = its current length, its K/V are appended to its pages, and
 * dev_logits[i, :] (fp32 [B, vocab]) receives the logits of the token after it.  Input tokens are
 * explicit so that a caller can feed back its own samples or force given tokens.
 * Workspace as for prefill with rows = B.  Errors as for prefill. */
int spiral_decode_step(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, int B,
                       const int32_t* dev_in_tokens, void* dev_ws, size_t ws_bytes,
                       float* dev_logits, void* stream);

/* One decode step fused with the actor's sampler: as spiral_decode_step followed by spiral_sample with generated
 * noise (seed, seq_id = host_seq_ids[i], step = host_steps[i]), bit for bit the same tokens, but the [B, vocab]
 * logits are never written: the LM head keeps the best score of every 128-column tile per row and a small
 * kernel picks the winner.  temperature == 0 is greedy decoding (host_steps may be NULL).  dev_out_tokens:
 * int32 [B]; it may be the same buffer as dev_in_tokens (free-running generation feeds the samples back).
 * Needs 16-bit weights repacked by spiral_model_repack, d_model % 128 == 0 and vocab % 16 == 0 (SHAPE error
 * otherwise; use the two separate calls then).  Workspace and other errors as spiral_decode_step. */
int spiral_decode_sample_step(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, int B,
                              const int32_t* dev_in_tokens, void* dev_ws, size_t ws_bytes, float temperature,
                              uint64_t seed, const int32_t* host_steps, int32_t* dev_out_tokens, void* stream);

/* ---- decode step without a workspace argument --------------------------------------------------
 * For callers that cannot allocate device memory or carry a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same step, same kernels and same results as
 * spiral_decode_step, but the workspace is the library's own scratch memory: a device array of
 * SPIRAL_STATIC_WORKSPACE_BYTES that every GPU the library runs on holds until the process ends.  Neither
 * this call nor anything it calls allocates or frees device memory.  A step that needs more
 * (spiral_workspace_bytes(m, B, longest context + 1) > spiral_static_workspace_bytes()) is rejected with
 * SPIRAL_ERR_OOM_KV and a message that says so; nothing is modified then.  All calls on one GPU share that
 * GPU's array: calls that overlap on one GPU (two streams, two threads, two models) race; calls in stream
 * order do not, and nothing has to be cleared between them (every part of the workspace a step reads it has
 * written before).  Other errors as spiral_decode_step. */
#define SPIRAL_STATIC_WORKSPACE_BYTES (16u << 20)
size_t spiral_static_workspace_bytes(void);
int spiral_decode_step_static(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, int B,
                              const int32_t* dev_in_tokens, float* dev_logits, void* stream);

/* ---- scoring pass (learner side) ---------------------------------------------------------------
 * The policy update of the paper (Alg. 1, last step; policy-gradient equation of Sec. 3) weights
 * log pi_theta(y_t | s_t) of every generated token with the RAE advantage of the player who produced it.
 * spiral_score runs the same packed forward as spiral_prefill (tokens are appended to the listed
 * sequences' caches, positions continue from their lengths, attention is causal over the whole history)
 * and returns, instead of last-token logits,
 *     dev_logp[r] = logit_r[dev_targets[r]] - logsumexp_v(logit_r[v])          fp32 [sum(host_lens)]
 * for every packed row r, 0 where dev_targets[r] < 0 (int32 [sum(host_lens)], ids < vocab; the usual
 * target of a row is the next token of its sequence).  The [rows, vocab] logits are never written.
 * 16-bit weights and d_model % 128 == 0 only.  Workspace and errors as for spiral_prefill. */
int spiral_score(spiral_model* m, spiral_kv_pool* p, const int32_t* host_seq_ids, const int32_t* host_lens,
                 int B, const int32_t* dev_tokens_packed, const int32_t* dev_targets, void* dev_ws,
                 size_t ws_bytes, float* dev_logp, void* stream);

/* Values of the objective for n tokens (device arrays; dev_mask int32 or NULL = all tokens count):
 *     dev_out2[0] = sum_t mask_t * min(r_t * A_t, clip(r_t, 1 - clip_eps, 1 + clip_eps) * A_t),  r_t = exp(new_t - old_t)
 *     dev_out2[1] = sum_t mask_t * A_t * new_t                                   (the REINFORCE sum of Sec. 3)
 * float64, fixed summation order, no normalisation by length (Sec. 3); clip_eps = 0.2 in the paper's
 * hyper-parameter table.  Errors: INVALID_ARG, HIP. */
int spiral_policy_objective(const float* dev_logp_new, const float* dev_logp_old, const float* dev_advantage,
                            const int32_t* dev_mask, long long n, float clip_eps, double* dev_out2, void* stream);

/* ---- sampling ---------------------------------------------------------------------------------
 * dev_out_tokens[i] = argmax_v( dev_logits[i,v] / temperature + g[i,v] ), lowest index on ties, in
 * fp32: an exact draw from softmax(logits / temperature) (Gumbel-max), the actor's untruncated
 * categorical (hyper-parameter table, App. D).  temperature == 0 selects greedy decoding (g = 0).
 * g is standard Gumbel noise -ln(-ln u): either read from dev_noise (fp32 [B, V], test mode) or,
 * when dev_noise is NULL, generated from the stateless counter generator
 *     mix(z): z^=z>>30; z*=0xBF58476D1CE4E5B9; z^=z>>27; z*=0x94D049BB133111EB; z^=z>>31   (mod 2^64)
 *     key = mix(mix(seed ^ 0x9E3779B97F4A7C15) + ((uint64)seq_id << 32 | step))
 *     r   = mix(key + v * 0x9E3779B97F4A7C15) >> 32 ;  u = ((r >> 9) + 0.5) * 2^-23
 * with seq_id = host_seq_ids[i] and step = host_steps[i] (both >= 0).  B <= SPIRAL_MAX_BATCH.
 * Errors: INVALID_ARG (null pointers, B or V < 1, temperature < 0 or not finite), HIP. */
int spiral_sample(const float* dev_logits, int B, int V, float temperature, uint64_t seed,
                  const int32_t* host_seq_ids, const int32_t* host_steps, const float* dev_noise,
                  int32_t* dev_out_tokens, void* stream);

/* ---- truncated sampling -----------------------------------------------------------------------
 * The evaluation-time decode setting of the paper (appendix "Evaluation Settings": temperature 0.6,
 * top-p 0.95); the actor's top-p = 1, top-k = -1 is the untruncated case and goes to spiral_sample.
 *     z_v = logit_v / temperature (fp32)
 *     top_k in (0, V): tau_k = the k-th largest z; keep z_v >= tau_k               (<= 0 or >= V: off)
 *     top_p in (0, 1): over the top-k survivors, walk z in descending order and stop where the running
 *                      sum of softmax(z) first reaches top_p; tau_p = that z; keep z_v >= tau_p  (1: off)
 *     token = argmax over { z_v >= max(tau_k, tau_p) } of z_v + g_v, lowest index on ties
 * Equal scores are kept or dropped together.  Noise g as in spiral_sample (dev_noise or generated).
 * dev_threshold_out (fp32 [B], may be NULL) receives the threshold max(tau_k, tau_p) of each row,
 * -inf when nothing was cut.  Running sums are 64-bit fixed point (2^-45 of the largest term), so
 * results are bit-reproducible.  temperature == 0 is greedy decoding (top_k, top_p ignored).
 * Errors: INVALID_ARG (as spiral_sample; top_p outside (0, 1]; threshold output with temperature 0), HIP. */
int spiral_sample_truncated(const float* dev_logits, int B, int V, float temperature, int top_k, float top_p,
                            uint64_t seed, const int32_t* host_seq_ids, const int32_t* host_steps,
                            const float* dev_noise, int32_t* dev_out_tokens, float* dev_threshold_out,
                            void* stream);
/* The same thresholds and the same draw (bit for bit) for long rows, in three sweeps of the logits instead of up to
 * nine and by several workgroups per row: dev_workspace (device memory, 256-byte aligned, contents undefined before and
 * after; calls that share it must be ordered on one stream) holds spiral_sample_truncated_workspace_bytes(B, V) bytes
 * (0 for an invalid B or V).  Rows shorter than 16384 entries, a call that cuts nothing, and single rows whose
 * scores are so crowded around the cut that more than 8192 of them fall within 1/128 of each other go through the
 * kernel of spiral_sample_truncated.  Errors: as spiral_sample_truncated; INVALID_ARG for a null, misaligned or
 * too small workspace. */
size_t spiral_sample_truncated_workspace_bytes(int B, int V);
int spiral_sample_truncated_ws(const float* dev_logits, int B, int V, float temperature, int top_k, float top_p,
                               uint64_t seed, const int32_t* host_seq_ids, const int32_t* host_steps,
                               const float* dev_noise, int32_t* dev_out_tokens, float* dev_threshold_out,
                               void* dev_workspace, size_t workspace_bytes, void* stream);

/* ---- measurement hooks (for benchmarks; not part of the method) --------------------------------
 * Between spiral_profile_begin and spiral_profile_end every launch of the chosen kernel class made
 * by spiral_prefill / spiral_decode_step on this model is bracketed by two HIP events on the call's
 * stream.  spiral_profile_end waits for the last event and reports the number of launches seen and
 * the sum of their durations in milliseconds.  At most max_launches launches are timed (further
 * ones run untimed).  Errors: INVALID_ARG (unknown class, max_launches < 1, begin while active,
 * end while inactive), HIP. */
enum spiral_kernel_class {
    SPIRAL_K_ATTN_DECODE = 0,   /* paged decode attention (without the merge of its partial results) */
    SPIRAL_K_ATTN_COMBINE,      /* merge of the partial results */
    SPIRAL_K_ATTN_PREFILL,
    SPIRAL_K_GEMM_QKV, SPIRAL_K_GEMM_O, SPIRAL_K_GEMM_GATE_UP, SPIRAL_K_GEMM_DOWN, SPIRAL_K_GEMM_LM_HEAD,
    SPIRAL_K_NORM,              /* embedding / residual-add + RMSNorm kernels */
    SPIRAL_K_QKV_POST,          /* bias | q/k norm + RoPE + KV append */
    SPIRAL_K_SAMPLE,            /* winner among the per-tile results of the fused LM head + sampler */
    SPIRAL_K_CLASSES
};
int spiral_profile_begin(spiral_model* m, int kernel_class, int max_launches);
int spiral_profile_end(spiral_model* m, double* host_total_ms, int* host_n_launches);
/* Yardstick for the memory-bound kernels: reads dev_buf (bytes >= 1 MiB, 16-byte aligned) `iters` times with a pure
 * streaming-load kernel shaped like the decode step's weight and K/V streams (3 workgroups per compute unit, eight
 * non-temporal 16-byte loads per lane in flight) and reports the mean milliseconds of one pass, measured with
 * HIP events on `stream`.  Unlike the rest of the library this call waits for its own work.  A buffer much smaller
 * than the last-level cache measures the cache, not HBM.  Errors: INVALID_ARG, HIP. */
int spiral_probe_stream_read(const void* dev_buf, size_t bytes, int iters, double* host_ms_per_pass, void* stream);

/* ---- role-conditioned advantage estimation (host only, float64) -------------------------------
 * Baselines b[game][role], role in {0,1}, start at 0 (Alg. 1, initialisation).  spiral_rae_update
 * processes n finished trajectories in array order; for trajectory i with game host_game_id[i] and
 * player-0 terminal reward host_r0[i] (player 1 receives -host_r0[i]: zero-sum), for role 0 then 1:
 *     b <- alpha * b + (1 - alpha) * R_role ;   adv[i][role] = R_role - b     (the updated b)
 * (Alg. 1, policy-optimisation loop; RAE equation, Sec. 3).  alpha in [0,1]; the paper uses 0.95.
 * host_adv: [n][2].  get/set copy the whole table [n_games][2].
 * Errors: INVALID_ARG (null, n < 0, game id out of range, alpha outside [0,1], non-finite reward);
 * on error nothing is modified. */
int  spiral_rae_create(int n_games, double alpha, spiral_rae** out);
int  spiral_rae_update(spiral_rae* r, const int32_t* host_game_id, const double* host_r0, int n,
                       double* host_adv);
int  spiral_rae_get(const spiral_rae* r, double* host_b);
int  spiral_rae_set(spiral_rae* r, const double* host_b);
void spiral_rae_free(spiral_rae* r);

#ifdef __cplusplus
}
#endif
#endif /* SPIRAL_H */
