/*
 * swift.h -- C ABI of the MI355X (gfx950) hot path of on-the-fly self-speculative
 * greedy decoding with a layer-skipping draft model.
 *
 * One decoding step of the method's acceleration phase (paper Section 4.2) is
 *     swift_draft_step  ->  swift_verify  ->  swift_accept
 * after one swift_prefill per input.  Plain autoregressive decoding of the
 * target model is the same loop with no draft tokens (swift_verify with k = 0).
 *
 * Conventions
 *  - Every function returns a status: SWIFT_OK (0) or a negative SWIFT_E* code.
 *    Nothing throws or aborts across this boundary.  On an error the decoding
 *    state (cache length, pending token, counters) is unchanged.
 *  - "host" pointers are ordinary process memory owned by the caller; they are
 *    only read or written during the call.  "device" pointers are HIP device
 *    memory of the current device.
 *  - The library allocates no device memory.  The caller hands it one device
 *    arena (size from swift_device_bytes) that holds the re-laid-out weights,
 *    the key/value cache, rotary tables and activations; the arena must stay
 *    alive and untouched by others until swift_destroy.
 *  - All GPU work is enqueued on the HIP stream given to swift_create; calls
 *    that return results to the host synchronise that stream before returning.
 *  - A context is not thread-safe; use one thread per context.
 *
 * Model (the paper names LLaMA-2 as backbone, Section 5.1): token embedding,
 * n_layers x [RMSNorm -> rotary (half-split pairs) causal attention with
 * n_q_heads query heads on n_kv_heads key/value heads -> residual add,
 * RMSNorm -> SwiGLU MLP -> residual add], final RMSNorm, untied LM head; no
 * biases.  Weights and the key/value cache are stored in `dtype`; the residual
 * stream, normalised activations, queries, attention probabilities, MLP
 * intermediates and logits are fp32 and every accumulation is fp32.
 *
 * Guarantee: a token's logits, and the keys and values it leaves in the cache, do
 * not depend on how many rows share its pass (one-row decoding, a draft pass, a
 * verify block or token tree of 2..32 rows): every kernel adds a row's products in the same
 * order.  Speculative greedy decoding therefore reproduces plain greedy decoding
 * of the same context exactly (paper Sections 1 and 3.1), not just up to
 * rounding.  Prefill blocks use an order of their own; both decoding modes share
 * the prefill.
 */
#ifndef SWIFT_H_
#define SWIFT_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SWIFT_OK 0
#define SWIFT_EINVAL (-1)    /* bad argument (null pointer, out-of-range value, unknown name, wrong size) */
#define SWIFT_ECAPACITY (-2) /* the call would write a cache slot >= max_seq, or the arena is too small */
#define SWIFT_ESTATE (-3)    /* call out of order (e.g. verify before prefill, accept before verify) */
#define SWIFT_EDEVICE (-4)   /* a HIP call failed; swift_last_error() has the text */

#define SWIFT_F32 0
#define SWIFT_BF16 1

/* Largest number of rows one verify block or token tree may hold (pending token + k drafts): k <=
 * SWIFT_MAX_BLOCK - 1.  The paper's maximum draft length is 25 (Appendix B.2): a chain block of 26 rows. */
#define SWIFT_MAX_BLOCK 32
/* Longest context window of a candidate evaluation (gamma of Section 4.1.2; Table 9 goes up to 128). */
#define SWIFT_MAX_WINDOW 128

typedef struct swift_model_config {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    int32_t max_seq;   /* capacity of the key/value cache in tokens */
    float rms_eps, rope_theta;
    int32_t dtype;     /* SWIFT_F32 or SWIFT_BF16: storage of weights and of the key/value cache */
} swift_model_config;

/* Counters behind the paper's metrics (Appendix B.3): mean generated length
 * M = emitted_by_verify / verify_passes, acceptance rate alpha = accepted / draft_passes. */
typedef struct swift_stats {
    int64_t draft_passes;      /* draft-model forward passes (= drafted tokens) */
    int64_t verify_passes;     /* target-model block passes */
    int64_t accepted;          /* draft tokens that passed verification */
    int64_t emitted_by_verify; /* tokens emitted by swift_accept (accepted + one target token per pass) */
    int64_t emitted_total;     /* emitted_by_verify + the token produced by swift_prefill */
} swift_stats;

typedef struct swift_ctx swift_ctx; /* opaque, owned by the library */

/* ---- host-only helpers (no GPU work; usable without a device) ------------------------------- */

/* Checks a configuration: positive sizes; head_dim 16, 32, 64 or 128; n_q_heads = 1, 2, 4 or 8
 * times n_kv_heads; hidden and ffn multiples of 8, vocab even, each at most 40704 (one fp32
 * activation row has to fit in LDS); known dtype. */
int swift_check_config(const swift_model_config *cfg);

/* Bytes of device memory swift_create needs for this configuration (weights in the library's
 * layout + key/value cache [layer][k|v][kv head][slot][head_dim] + tables + activations). */
int swift_device_bytes(const swift_model_config *cfg, uint64_t *bytes);

/* Expected wall-time speedup of the acceleration phase (Appendix B.3, Eq. 6):
 * M * alpha / ((M - 1) * c + alpha), c = cost of a draft pass relative to a target pass. */
double swift_expected_speedup(double mean_generated_length, double acceptance_rate, double cost_coefficient);

/* Greedy prefix acceptance (Section 4.2; draft-then-verify under greedy decoding): the largest
 * m <= k with draft[r] == target[r] for all r < m, where draft[r] is the (r+1)-th draft token and
 * target[r] the target model's arg-max after block row r.  Both arrays: host, k entries read. */
int swift_match_prefix(const int32_t *draft, const int32_t *target, int k);

/* Bytes the method has to move from HBM for ONE forward pass (weights of the non-skipped sublayers
 * and the LM head once, key/value slots [0, n_ctx) of the non-skipped attention sublayers, embedding
 * rows, key/value writes of `rows` rows).  skip_mask: host, uint8[2*n_layers] or NULL (= full model). */
int swift_pass_bytes(const swift_model_config *cfg, const uint8_t *skip_mask, int n_ctx, int rows, uint64_t *bytes);

/* Text of the last error of the calling thread ("" if none).  Owned by the library. */
const char *swift_last_error(void);

/* ---- context ------------------------------------------------------------------------------- */

/* Creates a context on the current HIP device.  device_mem: device arena of device_bytes bytes
 * (>= swift_device_bytes, 256-byte aligned).  hip_stream: a hipStream_t (NULL = default stream).
 * Builds the rotary cos/sin tables (angles in fp64 on the host, rounded to fp32). */
int swift_create(const swift_model_config *cfg, void *device_mem, uint64_t device_bytes, void *hip_stream,
                 swift_ctx **out);
int swift_destroy(swift_ctx *ctx);

/* Copies one tensor into the arena, converting to the library's layout.  data: host OR device
 * pointer, row-major [out][in], n_elems elements of type `dtype`, which must equal the model's
 * dtype for matrices and be SWIFT_F32 for the RMSNorm gains.  Names: "embed" [vocab][hidden],
 * "lm_head" [vocab][hidden], "final_norm" [hidden], and for layer i: "l<i>.attn_norm" [hidden],
 * "l<i>.wq" [n_q*d][hidden], "l<i>.wk", "l<i>.wv" [n_kv*d][hidden], "l<i>.wo" [hidden][n_q*d],
 * "l<i>.mlp_norm" [hidden], "l<i>.wg", "l<i>.wu" [ffn][hidden], "l<i>.wd" [hidden][ffn].
 * The caller's buffer may be freed after the call returns.  All tensors must be loaded before
 * swift_prefill (else SWIFT_ESTATE). */
int swift_load_tensor(swift_ctx *ctx, const char *name, const void *data, int dtype, int64_t n_elems);

/* ---- the decoding path ----------------------------------------------------------------------- */

/* Prefill: the full model over prompt[0..n_prompt) (host) at positions 0..n_prompt-1; fills the
 * key/value cache; *first_token = arg-max of the last row, which becomes the pending token (the
 * last emitted token, not yet in the cache).  Resets counters and state.  Needs
 * 1 <= n_prompt < max_seq. */
int swift_prefill(swift_ctx *ctx, const int32_t *prompt, int n_prompt, int32_t *first_token);

/* Drafting (Section 4.2, Eq. 5 with early stopping): starting from the pending token at position
 * n = cache length, runs the draft model -- the target model with the sublayers in skip_mask
 * bypassed (Section 3.1) -- autoregressively for up to max_k tokens.  Draft token j is the arg-max
 * of the draft logits (lowest index on ties), draft_conf[j-1] its top-1 softmax probability; drafting
 * stops after the first token whose confidence is < conf_threshold (that token is kept).
 * skip_mask: host, uint8[2*n_layers], entry 2l = attention sublayer of layer l, 2l+1 = its MLP,
 * non-zero = skipped.  A skipped sublayer leaves the residual stream unchanged and writes no
 * key/value.  Draft keys/values go to slots n.. of the non-skipped attention sublayers.
 * A verification that has not been accepted yet is cancelled (its swift_accept then fails with
 * SWIFT_ESTATE): the draft overwrites cache slots that verification wrote.
 * draft_tokens / draft_conf: host arrays of max_k entries; *k_out in [0, max_k].
 * Needs 0 <= max_k <= SWIFT_MAX_BLOCK - 1 and n + max_k + 1 <= max_seq (SWIFT_ECAPACITY). */
int swift_draft_step(swift_ctx *ctx, const uint8_t *skip_mask, int max_k, float conf_threshold,
                     int32_t *draft_tokens, float *draft_conf, int *k_out);

/* Parallel candidate evaluation of the paper's optimisation phase (Section 4.1.2, Eq. 3 and Eq. 4):
 * a candidate draft model (skipped set skip_mask, as in swift_draft_step) predicts each of the last
 * gamma generated tokens from the context before it, in one block pass that reuses the target
 * model's cached keys and values.  window (host, gamma + 1 ids): the tokens at positions
 * n - gamma .. n of the sequence, i.e. the last gamma committed tokens and then the pending token
 * (n = cache length).  Row i reads window[i] at position n - gamma + i and attends the cache slots
 * 0 .. n - gamma + i as they are (nothing is written; keys and values of the rows are not computed);
 * predicted[i] (host, gamma ids, may be NULL) = its arg-max, the prediction of window[i + 1].
 * *n_match = number of i with predicted[i] == window[i + 1]; matchness = *n_match / gamma.
 * 1 <= gamma <= SWIFT_MAX_WINDOW (the largest context window of the paper's Table 9; a window of more
 * than 64 tokens runs as one macro block of two 64-row sub-blocks on bf16 models, as two blocks
 * otherwise) and gamma <= n, else SWIFT_EINVAL / SWIFT_ESTATE.  Cache, cache length, pending
 * token, outstanding draft/verify state and statistics are left unchanged. */
int swift_eval_mask(swift_ctx *ctx, const uint8_t *skip_mask, const int32_t *window, int gamma,
                    int32_t *predicted, int *n_match);

/* ---- Optimisation phase on top of swift_eval_mask (Sections 4.1.1 and 4.1.2, Eq. 2; Appendix B.2).
 * Host logic only.  One swift_opt_step before a decoding step: step 1 scores the uniform initial
 * skipping pattern (the skipped sublayers spread evenly over the eligible ones), every later step a
 * random-search candidate with exactly round(skip_ratio * n_sublayers) eligible sublayers skipped;
 * the candidate replaces the retained set if its matchness on the current window is strictly higher.
 * The phase is finished when max_steps steps are done, or max_stale steps in a row brought no
 * improvement, or the best matchness exceeds stop_matchness (the paper: 1000, 300, 0.95).
 * Random search draws from a counter-based generator keyed by (seed, step): candidates do not depend
 * on what was evaluated before.  mix64(x): z = x + 0x9E3779B97F4A7C15; z = (z ^ z >> 30) *
 * 0xBF58476D1CE4E5B9; z = (z ^ z >> 27) * 0x94D049BB133111EB; z ^ z >> 31.  key = mix64(mix64(seed ^
 * 0x53574946544F5054) + step); draw j = mix64(key + j); partial Fisher-Yates over the eligible list
 * in index order: entry j is swapped with entry j + draw_j mod (E - j), j < n_skip.
 * Bayesian optimisation is not built; swift_opt_set_suggester lets a caller take every interval-th
 * step (the paper's beta = 25) with a candidate of its own (return 0 and fill `candidate`; any other
 * return falls back to random search). */
typedef struct {
    int n_sublayers;        /* 2 * n_layers: attention and MLP sublayers, index order as in skip masks */
    double skip_ratio;      /* r in [0, 1] */
    int max_steps;          /* S >= 1 */
    int max_stale;          /* >= 1 */
    double stop_matchness;
    uint64_t seed;
} swift_opt_config;
typedef struct swift_opt swift_opt; /* opaque; owned by the library */
typedef int (*swift_suggest_fn)(void *user, int step, const uint8_t *best_mask, double best_matchness, int n_sublayers,
                                uint8_t *candidate);
/* eligible: host, n_sublayers bytes, 1 = may be skipped (NULL: all).  SWIFT_EINVAL if the ratio asks
 * for more skipped sublayers than are eligible. */
int swift_opt_create(const swift_opt_config *cfg, const uint8_t *eligible, swift_opt **out);
int swift_opt_destroy(swift_opt *opt);
int swift_opt_initial_mask(const swift_opt *opt, uint8_t *mask);          /* mask: host, n_sublayers bytes */
int swift_opt_candidate(const swift_opt *opt, int step, uint8_t *mask);   /* the random-search candidate of a step */
int swift_opt_set_suggester(swift_opt *opt, swift_suggest_fn fn, void *user, int interval);
/* window, gamma: as for swift_eval_mask.  Outputs (host; each may be NULL): the step's candidate and its
 * matchness, the retained set and its matchness, finished (0/1).  SWIFT_ESTATE once finished; SWIFT_EINVAL
 * if the optimiser's n_sublayers is not twice the context's layer count; errors of swift_eval_mask are
 * passed on and leave the optimiser unchanged. */
int swift_opt_step(swift_ctx *ctx, swift_opt *opt, const int32_t *window, int gamma, uint8_t *candidate,
                   double *candidate_matchness, uint8_t *best_mask, double *best_matchness, int *finished);

/* Verification (Sections 1, 3.1: drafts are validated in parallel by the full model): the target
 * model over the k+1 rows tokens[0..k] (host; tokens[0] must be the pending token) at positions
 * n..n+k, row i attending slots 0..n+i; target keys/values overwrite slots n..n+k of every layer.
 * target_tokens[i] (host, k+1 entries) = arg-max of row i.  logits_out: NULL, or host fp32
 * [k+1][vocab].  k = 0 is one step of plain autoregressive decoding.
 * Needs 0 <= k <= SWIFT_MAX_BLOCK - 1 and n + k + 1 <= max_seq. */
int swift_verify(swift_ctx *ctx, const int32_t *tokens, int k, int32_t *target_tokens, float *logits_out);

/* swift_verify for callers that must not allocate (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same kernels and the same results bit for bit, but their scratch
 * memory (arrival counters and partial sums of projections that split K over workgroups, partial results
 * of attention split over the cache length) lies in a device array of SWIFT_STATIC_SCRATCH_BYTES that is
 * part of the library's code object instead of in the context's arena.  The call allocates and frees
 * nothing, on the device or the pinned host side, and creates no events (per-class timing is off
 * during it).  Every GPU the library runs on holds that array from the first use until the process ends.
 * A block whose partial results do not fit (many query heads times many block rows times many cache
 * ranges: e.g. more than 7 rows of a 64-head model with a cache of thousands of slots) is refused with
 * SWIFT_ECAPACITY and a message that says so, before anything is launched; swift_verify takes it.
 * All contexts of a process share one array per GPU, and it keeps the last call's contents: calls that
 * overlap on one GPU (two streams, two threads) race; one call at a time per GPU.
 * State changes, errors and the following swift_accept are exactly those of swift_verify. */
#define SWIFT_STATIC_SCRATCH_BYTES (32u << 20)
int swift_verify_static(swift_ctx *ctx, const int32_t *tokens, int k, int32_t *target_tokens, float *logits_out);

/* Acceptance + roll-back after a swift_verify: m = swift_match_prefix(tokens[1..k], targets);
 * emitted (host, capacity >= k+1) receives the m accepted draft tokens followed by the target's own
 * token; *n_emitted = m + 1; the cache length becomes n + m + 1 and the last emitted token becomes
 * the pending token.  Slots at or beyond the new cache length are don't-care from here on. */
int swift_accept(swift_ctx *ctx, int32_t *emitted, int *n_emitted);

/* ---- dynamic verification (Section 4.2, second strategy of the inference phase) ----------------
 * Each draft position keeps its top candidates, the fewer the more confident the draft model is, and the
 * target model verifies all of them in one block whose rows form a token tree.
 * Readings (the paper gives the bands and the idea, not the tree's shape): only the first candidate of
 * a position (the greedy draft token) is continued by the draft model, so a position's other candidates
 * are leaves; a block holds at most SWIFT_MAX_BLOCK rows (pending token + all candidates). */
#define SWIFT_TOPK 10
/* Candidates kept for a position drafted with confidence p: 10, 5, 3, 1 for p in (0, 0.5], (0.5, 0.8],
 * (0.8, 0.95], (0.95, 1]. */
int swift_topk_width(float p);

/* swift_draft_step that also keeps candidates: position j = 1..*k_out gets width[j-1] =
 * min(swift_topk_width(p_j), max_width, rows still free in the block) tokens (a block holds at most
 * min(SWIFT_MAX_BLOCK, max_seq - n) rows: every row takes a cache slot of its own) in
 * tokens[(j-1)*SWIFT_TOPK ..] (host, [max_k][SWIFT_TOPK]; largest logit first, equal logits in id order;
 * the first is the draft token the next position continues from).  Drafting ends as in swift_draft_step, or
 * when the block is full.  draft_conf, width: host, max_k entries.  max_width >= 1 (1: the plain chain).
 * Needs 0 <= max_k <= SWIFT_MAX_BLOCK - 1 and n < max_seq (SWIFT_ECAPACITY). */
int swift_draft_step_topk(swift_ctx *ctx, const uint8_t *skip_mask, int max_k, float conf_threshold, int max_width,
                          int32_t *tokens, float *draft_conf, int *width, int *k_out);

/* Verification of a token tree in one block of the target model.  tokens (host): row 0 = the pending
 * token, then the width[0] candidates of level 1, the width[1] of level 2, ... (`levels` levels; rows =
 * 1 + sum width <= SWIFT_MAX_BLOCK; 1 <= width[j] <= SWIFT_TOPK).  A row of level j is computed at sequence
 * position n + j; it attends the committed slots 0..n-1, row 0, the first rows of levels 1..j-1 and itself;
 * its keys/values go to cache slot n + (row index).  target_tokens (host, one per row) = arg-max of each
 * row: the target's next token after the path that ends in that row.  logits_out: NULL, or host fp32
 * [rows][vocab].  Every row's result equals, bit for bit, that of the same path verified as a chain by
 * swift_verify.  levels = 0 is one step of plain decoding.  Errors as swift_verify. */
int swift_verify_tree(swift_ctx *ctx, const int32_t *tokens, const int *width, int levels, int32_t *target_tokens,
                      float *logits_out);

/* Acceptance after a swift_verify_tree: starting with the target's token after the pending token, a level
 * is accepted if one of its candidates equals the target's token for the path so far (the path goes on
 * only through a level's first candidate).  emitted (host, capacity >= levels + 1) receives the m accepted
 * candidates and the target's own next token; *n_emitted = m + 1.  The accepted rows' keys/values are moved
 * to slots n+1..n+m of every layer (device copy, stream-ordered), the cache length becomes n + m + 1 and
 * the last emitted token the pending token.  SWIFT_ESTATE without a preceding swift_verify_tree. */
int swift_accept_tree(swift_ctx *ctx, int32_t *emitted, int *n_emitted);

/* ---- speculative sampling (Section 5.1 and Appendix B.2: speculative sampling is the acceptance rule;
 * the sampled runs use temperature 0.6 and top-p 0.95) --------------------------------------------
 * Tokens are drawn from W(logits) = softmax(logits / temperature) cut to its nucleus and renormalised.
 * Nucleus: the tokens whose probability is at least t*, the largest probability value t for which the
 * tokens with probability >= t together reach top_p (tokens as probable as the last one needed all stay;
 * top_p >= 1 keeps everything).  A draw with the uniform u in [0, 1) takes the first token id j with
 * W_0 + .. + W_j > u * (W_0 + .. + W_{V-1}).  The library draws no random numbers: the caller passes the
 * uniforms (SWIFT_EINVAL outside [0, 1)), so a run is reproducible and testable against other code.
 * Arithmetic in fp32; temperature > 0 and top_p > 0. */

/* swift_prefill, then the first token is drawn with u from W of the last prompt row's logits. */
int swift_prefill_sample(swift_ctx *ctx, const int32_t *prompt, int n_prompt, float temperature, float top_p, float u,
                         int32_t *first_token);

/* swift_draft_step with sampled draft tokens: draft token j is drawn with u[j-1] (host, max_k entries) from
 * q_j = W(draft logits of position j), which stays on the device for the acceptance test.  draft_conf and
 * the early stop use the top-1 probability of the plain softmax, as in swift_draft_step (the paper does not
 * say what the confidence is when sampling). */
int swift_draft_step_sample(swift_ctx *ctx, const uint8_t *skip_mask, int max_k, float conf_threshold,
                            float temperature, float top_p, const float *u, int32_t *draft_tokens, float *draft_conf,
                            int *k_out);

/* Verification and acceptance in one call.  tokens[0..k] (host): the pending token and the first k draft
 * tokens of the preceding swift_draft_step_sample (SWIFT_ESTATE / SWIFT_EINVAL otherwise).  The target
 * model runs over the block as in swift_verify; p_i = W(logits of row i-1).  Draft token x_i is kept iff
 * u_accept[i-1] * q_i(x_i) < p_i(x_i), i.e. with probability min(1, p_i(x_i) / q_i(x_i)); the first token not
 * kept is replaced by a draw with u_final from max(0, p_i - q_i) renormalised and ends the step; if all k
 * are kept, one more token is drawn with u_final from p_{k+1}.  emitted (host, capacity >= k+1), *n_emitted
 * = kept + 1; cache length, pending token and statistics change as after swift_accept.  k = 0: one step
 * of plain sampling.  probs_out: NULL, or host fp32 [k+1][vocab] = p_1 .. p_{k+1}.
 * u_accept: host, k entries. */
int swift_verify_sample(swift_ctx *ctx, const int32_t *tokens, int k, float temperature, float top_p,
                        const float *u_accept, float u_final, int32_t *emitted, int *n_emitted, float *probs_out);

/* Sets the cache length to new_cache_len <= current (no data is touched) and makes
 * `pending_token` the pending token.  For callers that manage acceptance themselves. */
int swift_rollback(swift_ctx *ctx, int new_cache_len, int32_t pending_token);

int swift_get_state(swift_ctx *ctx, int *cache_len, int32_t *pending_token);
/* The configuration the context was created with. */
int swift_get_config(swift_ctx *ctx, swift_model_config *out);
int swift_get_stats(swift_ctx *ctx, swift_stats *out);

/* ---- test and measurement hooks -------------------------------------------------------------- */

/* NaN-fills every key/value slot at or beyond the cache length (results must not change). */
int swift_debug_poison_kv(swift_ctx *ctx);
/* Copies logits row `row` of the most recent pass (draft: row 0) to out (host fp32 [vocab]). */
int swift_debug_read_logits(swift_ctx *ctx, int row, float *out);
/* Copies slot `pos` of layer `layer` to k_out / v_out (host fp32 [n_kv_heads*head_dim] each). */
int swift_debug_read_kv(swift_ctx *ctx, int layer, int pos, float *k_out, float *v_out);

/* Names the attention kernel instance a block of `rows` rows would take in this context at its present
 * cache length (tree != 0: the rows of a token tree), e.g. "split<bf16, group 1, rows 3>": kernel family,
 * storage type, query heads per key/value head, block rows that share a workgroup's key/value loads.
 * out: host, capacity bytes, NUL-terminated.  Host only; for tests that must know what they covered. */
int swift_debug_attn_path(swift_ctx *ctx, int rows, int tree, char *out, int capacity);

/* Kernel classes for per-kernel timing. */
#define SWIFT_KC_QKV 0      /* RMSNorm + fused Q/K/V projection + rotation + cache append */
#define SWIFT_KC_ATTN 1     /* attention over the cache (+ split combine) */
#define SWIFT_KC_OPROJ 2    /* output projection + residual add */
#define SWIFT_KC_GATEUP 3   /* RMSNorm + gate/up projections + SwiGLU */
#define SWIFT_KC_DOWN 4     /* down projection + residual add */
#define SWIFT_KC_LMHEAD 5   /* final RMSNorm + LM head + arg-max/softmax partials */
#define SWIFT_KC_OTHER 6    /* embedding gather, arg-max finalisation */
#define SWIFT_KC_COUNT 7

/* Overrides the launch shape of the tiled single-row projection kernel of one class: wavefronts
 * that share a 16-row group (0 = automatic, else 1, 2, 4 or 8) and workgroups (0 = automatic).
 * Results do not depend on it bit for bit only within one setting; it exists for tuning runs. */
int swift_debug_tune(swift_ctx *ctx, int kernel_class, int waves_per_row_group, int workgroups);

/* How swift_prefill walks a prompt on bf16 models (tuning and test runs; every setting gives results within the
 * library's tolerance, not the same bits).  sub_blocks: 0 = the default (macro blocks of up to 8 sub-blocks of 64
 * rows per sweep over the weights), 1..8 = macro blocks of at most that many sub-blocks, -1 = one 64-row block per
 * sweep.  tiling: 0 = automatic, else the workgroup tile of the blocked matrix product: 1..4 = 64, 128, 192 or 256
 * weight rows x two sub-blocks, 5 / 6 = 128 / 256 weight rows x one sub-block. */
int swift_debug_prefill(swift_ctx *ctx, int sub_blocks, int tiling);

/* Turns per-launch timing of one kernel class on (kernel_class in [0, SWIFT_KC_COUNT)) or off (-1).
 * While on, every launch of that class is bracketed by HIP events on the context's stream. */
int swift_profile_class(swift_ctx *ctx, int kernel_class);
/* Synchronises, then returns the launches recorded since the last call, their summed duration in
 * milliseconds and the summed algorithmic HBM bytes of those launches; resets the record. */
int swift_profile_read(swift_ctx *ctx, int64_t *launches, double *total_ms, uint64_t *total_bytes);

#ifdef __cplusplus
}
#endif
#endif /* SWIFT_H_ */
