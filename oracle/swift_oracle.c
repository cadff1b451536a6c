/*
 * swift_oracle.c -- CPU oracle for layer-skipping self-speculative greedy decoding.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is checked against.  Nothing in the product path may link, load
 * or call it; only the tests, the smoke check and the benchmark's CPU-baseline
 * leg do.  It shares no code with the HIP library.
 *
 * What it computes
 *   - The target model M_T: a LLaMA-style decoder (the paper names LLaMA-2 as
 *     its backbone, Section 5.1): token embedding, L layers of
 *     [pre-RMSNorm -> rotary multi-head / grouped-query causal attention ->
 *     residual add] and [pre-RMSNorm -> SwiGLU MLP -> residual add], a final
 *     RMSNorm and an untied LM head.  No biases.
 *   - The draft model M_D: the same network with the sublayers named by the
 *     skipped-layer set z bypassed (Section 3.1: z in {0,1}^L with L counting
 *     attention and MLP sublayers separately).  A skipped sublayer leaves the
 *     residual stream untouched and writes no key/value.
 *   - One decoding step of the acceleration phase (Section 4.2): greedy
 *     autoregressive drafting (Eq. 5) with confidence p_j = max softmax and
 *     early stop when p_j < eps, verification of [pending, y'_1..y'_k] by the
 *     full model in one causal block, acceptance of the longest matching
 *     prefix plus the target's own next token, and roll-back of the cache
 *     length.
 *   - Plain greedy autoregressive decoding (the definition the method must
 *     reproduce token for token), a brute-force forward without any cache,
 *     and the expected-speedup closed form (Appendix B.3, Eq. 6).
 *   - Dynamic verification (Section 4.2, strategy 2): every draft position is
 *     widened to its top-k draft predictions, k = 10, 5, 3, 1 for a confidence in
 *     (0, 0.5], (0.5, 0.8], (0.8, 0.95], (0.95, 1]; all candidates are verified
 *     in one block whose rows attend the committed context, their ancestors in
 *     the token tree and themselves; the longest accepted path is kept and its
 *     keys/values are moved to consecutive cache slots.
 *   - Parallel candidate evaluation of the optimisation phase (Section 4.1.2,
 *     Eq. 3 and Eq. 4): a candidate draft model predicts each of the last
 *     gamma generated tokens from the context before it, reusing the target
 *     model's cached keys and values, and the matchness score counts the
 *     predictions that equal the generated tokens.
 *   - The random-search part of the layer set suggestion (Section 4.1.2,
 *     Eq. 2 with a fixed skip ratio r) and the bookkeeping of the optimisation
 *     phase: the uniform initial skipping pattern (Section 4.1.1), one
 *     candidate per optimisation step, the best-scoring candidate retained,
 *     and the termination rules of Appendix B.2 (step limit, no improvement
 *     for a number of steps, matchness above a bound).  Bayesian optimisation
 *     is not part of it.
 *
 * Arithmetic
 *   Every floating-point step is carried out in fp64.  Rounding happens only
 *   where the data format fixes it: weights arrive already rounded to their
 *   storage type (fp32 or bf16); keys (after the rotation) and values are
 *   rounded to the cache's storage type when they are written, taking that
 *   decision the way an fp32 kernel would (fp64 -> fp32 -> storage type);
 *   rotary cos/sin are rounded to fp32; logits are rounded to fp32 before the
 *   arg-max so that ties are decided in the precision the logits are reported
 *   in.  Each dot product runs over its index in increasing order with one
 *   accumulator, attention runs over cache slots in increasing order, and a
 *   block of rows is simply the single-row forward called once per row, so a
 *   token's logits are bit-identical whether it is computed alone or inside a
 *   verify block.  Threads split output rows only, never a reduction, so the
 *   result does not depend on the thread count.
 *
 * Parity pins (tests/test_oracle_*.py): speculative output == autoregressive
 * output for many masks / draft lengths / thresholds; cached forward ==
 * brute-force forward; closed forms for the all-skipped draft, single-slot
 * and equal-key attention, uniform logits; RoPE worked example and
 * relative-position property; RMSNorm invariances; Eq. 6 against the values
 * printed in the paper's Table 4; candidate evaluation: the empty skipped set
 * scores gamma out of gamma on the model's own greedy output, the all-skipped
 * set has a closed form, rows do not depend on later cache slots, the decoding
 * state is left untouched.
 * Parity unpinned: behaviour on trained weights (acceptance rates, M, the
 * measured speedups) -- needs checkpoints and datasets that are not available.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORA_OK 0
#define ORA_EINVAL -1
#define ORA_ECAPACITY -2
#define ORA_ESTATE -3

#define ORA_F32 0
#define ORA_BF16 1
#define ORA_MAX_BLOCK 64
#define ORA_TREE_ROWS 32 /* rows of a token tree block: the pending token + all candidates (room for the
                            paper's maximum draft length of 25, Appendix B.2) */
#define ORA_TOPK 10      /* widest candidate set of one draft position */

typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab, max_seq;
    double rms_eps, rope_theta;
    int32_t kv_dtype; /* ORA_F32 or ORA_BF16: storage type of the key/value cache */
} ora_config;

typedef struct {
    const void *p; /* borrowed, row-major [out][in] */
    int dtype;
    int64_t n;
} ora_tensor;

typedef struct {
    ora_tensor attn_norm, wq, wk, wv, wo, mlp_norm, wg, wu, wd;
} ora_layer;

typedef struct ora_model {
    ora_config c;
    ora_tensor embed, final_norm, lm_head;
    ora_layer *layers;
    float *kcache, *vcache; /* [L][max_seq][n_kv*d]; values already rounded to kv_dtype */
    int threads;
    /* decoding state */
    int n;        /* cache length: slots [0,n) hold committed target keys/values */
    int pending;  /* last emitted token, not yet in the cache; -1 before prefill */
    int k_draft;  /* draft tokens of the current step (-1: none drafted) */
    int32_t draft[ORA_MAX_BLOCK];
    int k_verify; /* k of the last verify (-1: none) */
    int32_t vtokens[ORA_MAX_BLOCK + 1];
    int32_t target[ORA_MAX_BLOCK + 1];
    /* token tree of the last dynamic verification (-1: none) */
    int tree_levels;
    int tree_width[ORA_TREE_ROWS];
    int32_t tree_tokens[ORA_TREE_ROWS], tree_target[ORA_TREE_ROWS];
    /* speculative sampling: the draft distributions of the current step, [ORA_TREE_ROWS][vocab] */
    double *qdist;
    int k_sampled; /* draft tokens drawn by the last ora_draft_step_sample (-1: none) */
    /* counters (Appendix B.3) */
    int64_t n_draft_passes, n_verify_passes, n_accepted, n_emitted;
} ora_model;

/* ---------------------------------------------------------------- helpers */

static inline float bf16_bits_to_float(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* fp32 -> bf16 by round-to-nearest-even, returned as the fp32 it represents */
static inline float round_to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return f; /* NaN stays NaN */
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return f;
}

static inline double tget(const ora_tensor *t, int64_t i) {
    if (t->dtype == ORA_F32) return (double)((const float *)t->p)[i];
    return (double)bf16_bits_to_float(((const uint16_t *)t->p)[i]);
}

/* y[o] = sum_{i=0..K-1} W[o][i] * x[i], i increasing, one fp64 accumulator */
static void matvec(const ora_model *m, const ora_tensor *W, int O, int K, const double *x, double *y) {
    (void)m;
#pragma omp parallel for schedule(static) num_threads(m->threads)
    for (int o = 0; o < O; ++o) {
        double acc = 0.0;
        if (W->dtype == ORA_F32) {
            const float *w = (const float *)W->p + (int64_t)o * K;
            for (int i = 0; i < K; ++i) acc += (double)w[i] * x[i];
        } else {
            const uint16_t *w = (const uint16_t *)W->p + (int64_t)o * K;
            for (int i = 0; i < K; ++i) acc += (double)bf16_bits_to_float(w[i]) * x[i];
        }
        y[o] = acc;
    }
}

/* RMSNorm: out_i = x_i * g_i / sqrt(mean_j x_j^2 + eps) */
void ora_rmsnorm(const double *x, const double *g, int n, double eps, double *out) {
    double ss = 0.0;
    for (int i = 0; i < n; ++i) ss += x[i] * x[i];
    double r = 1.0 / sqrt(ss / (double)n + eps);
    for (int i = 0; i < n; ++i) out[i] = x[i] * r * g[i];
}

static void rmsnorm_t(const double *x, const ora_tensor *g, int n, double eps, double *out) {
    double ss = 0.0;
    for (int i = 0; i < n; ++i) ss += x[i] * x[i];
    double r = 1.0 / sqrt(ss / (double)n + eps);
    for (int i = 0; i < n; ++i) out[i] = x[i] * r * tget(g, i);
}

/* Rotary embedding of one head vector at absolute position pos, in place.
 * Pairs (i, i + d/2); frequency theta^(-2i/d); angle pos * frequency;
 * (a, b) -> (a cos - b sin, b cos + a sin).  cos/sin are rounded to fp32. */
void ora_rope(double *v, int d, int pos, double theta) {
    int half = d / 2;
    for (int i = 0; i < half; ++i) {
        double freq = pow(theta, -2.0 * (double)i / (double)d);
        double ang = (double)pos * freq;
        double c = (double)(float)cos(ang), s = (double)(float)sin(ang);
        double a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

static inline float round_kv(const ora_config *c, double x) {
    float f = (float)x;
    return c->kv_dtype == ORA_BF16 ? round_to_bf16(f) : f;
}

/* One query head against n_ctx cached slots: softmax(q.k_u / sqrt(d)) . v_u.
 * kc / vc point at slot 0 of the right KV head; consecutive slots are `stride` apart. */
void ora_attend(const double *q, const float *kc, const float *vc, int64_t stride, int n_ctx, int d,
                double *out) {
    double *s = (double *)malloc(sizeof(double) * (size_t)n_ctx);
    double scale = 1.0 / sqrt((double)d), mx = -INFINITY;
    for (int u = 0; u < n_ctx; ++u) {
        double acc = 0.0;
        const float *kr = kc + (int64_t)u * stride;
        for (int i = 0; i < d; ++i) acc += q[i] * (double)kr[i];
        s[u] = acc * scale;
        if (s[u] > mx) mx = s[u];
    }
    double den = 0.0;
    for (int u = 0; u < n_ctx; ++u) {
        s[u] = exp(s[u] - mx);
        den += s[u];
    }
    for (int i = 0; i < d; ++i) out[i] = 0.0;
    for (int u = 0; u < n_ctx; ++u) {
        double a = s[u] / den;
        const float *vr = vc + (int64_t)u * stride;
        for (int i = 0; i < d; ++i) out[i] += a * (double)vr[i];
    }
    free(s);
}

/* SwiGLU gate: silu(g) * u with silu(z) = z / (1 + exp(-z)) */
double ora_swiglu(double g, double u) { return g / (1.0 + exp(-g)) * u; }

/* Greedy choice and confidence from a logits row.
 * token = lowest index attaining the maximum of the fp32-rounded logits;
 * conf  = max softmax = 1 / sum_i exp(l_i - l_max)  (temperature 1). */
void ora_argmax_conf(const double *logits, int n, int32_t *token, double *conf) {
    int best = 0;
    float bv = (float)logits[0];
    for (int i = 1; i < n; ++i) {
        float v = (float)logits[i];
        if (v > bv) {
            bv = v;
            best = i;
        }
    }
    double den = 0.0;
    for (int i = 0; i < n; ++i) den += exp((double)(float)logits[i] - (double)bv);
    *token = best;
    if (conf) *conf = 1.0 / den;
}

/* Expected wall-time speedup of the acceleration phase (Appendix B.3, Eq. 6):
 * M tokens per target pass cost one target pass plus (M-1)/alpha draft passes
 * of relative cost c each. */
double ora_expected_speedup(double M, double alpha, double c) { return M * alpha / ((M - 1.0) * c + alpha); }

/* Longest accepted prefix: largest m <= k with draft[r] == target[r] for all r < m
 * (draft[r] is y'_{r+1}; target[r] is the full model's greedy token after row r). */
int ora_match_prefix(const int32_t *draft, const int32_t *target, int k) {
    int m = 0;
    while (m < k && draft[m] == target[m]) ++m;
    return m;
}

/* ---------------------------------------------------------------- model */

int ora_create(const ora_config *c, ora_model **out) {
    if (!c || !out) return ORA_EINVAL;
    if (c->n_layers <= 0 || c->hidden <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 ||
        (c->head_dim & 1) || c->ffn <= 0 || c->vocab <= 0 || c->max_seq <= 0 ||
        c->n_q_heads % c->n_kv_heads != 0 || (c->kv_dtype != ORA_F32 && c->kv_dtype != ORA_BF16))
        return ORA_EINVAL;
    ora_model *m = (ora_model *)calloc(1, sizeof(ora_model));
    m->c = *c;
    m->layers = (ora_layer *)calloc((size_t)c->n_layers, sizeof(ora_layer));
    size_t kvn = (size_t)c->n_layers * c->max_seq * c->n_kv_heads * c->head_dim;
    m->kcache = (float *)calloc(kvn, sizeof(float));
    m->vcache = (float *)calloc(kvn, sizeof(float));
    m->threads = 1;
    m->pending = -1;
    m->k_draft = -1;
    m->k_verify = -1;
    m->tree_levels = -1;
    m->k_sampled = -1;
    *out = m;
    return ORA_OK;
}

void ora_destroy(ora_model *m) {
    if (!m) return;
    free(m->layers);
    free(m->kcache);
    free(m->vcache);
    free(m->qdist);
    free(m);
}

void ora_set_threads(ora_model *m, int t) { m->threads = t < 1 ? 1 : t; }

int ora_threads_available(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Borrow a tensor.  name: "embed", "final_norm", "lm_head",
 * "l<i>.{attn_norm,wq,wk,wv,wo,mlp_norm,wg,wu,wd}"; row-major [out][in]. */
int ora_set_tensor(ora_model *m, const char *name, const void *data, int dtype, int64_t n) {
    if (!m || !name || !data || (dtype != ORA_F32 && dtype != ORA_BF16)) return ORA_EINVAL;
    const ora_config *c = &m->c;
    int64_t H = c->hidden, Q = (int64_t)c->n_q_heads * c->head_dim, KV = (int64_t)c->n_kv_heads * c->head_dim,
            F = c->ffn, V = c->vocab;
    ora_tensor t = {data, dtype, n};
    ora_tensor *dst = NULL;
    int64_t want = -1;
    if (!strcmp(name, "embed")) dst = &m->embed, want = V * H;
    else if (!strcmp(name, "final_norm")) dst = &m->final_norm, want = H;
    else if (!strcmp(name, "lm_head")) dst = &m->lm_head, want = V * H;
    else if (name[0] == 'l') {
        char *end;
        long l = strtol(name + 1, &end, 10);
        if (end == name + 1 || *end != '.' || l < 0 || l >= c->n_layers) return ORA_EINVAL;
        const char *f = end + 1;
        ora_layer *y = &m->layers[l];
        if (!strcmp(f, "attn_norm")) dst = &y->attn_norm, want = H;
        else if (!strcmp(f, "wq")) dst = &y->wq, want = Q * H;
        else if (!strcmp(f, "wk")) dst = &y->wk, want = KV * H;
        else if (!strcmp(f, "wv")) dst = &y->wv, want = KV * H;
        else if (!strcmp(f, "wo")) dst = &y->wo, want = H * Q;
        else if (!strcmp(f, "mlp_norm")) dst = &y->mlp_norm, want = H;
        else if (!strcmp(f, "wg")) dst = &y->wg, want = F * H;
        else if (!strcmp(f, "wu")) dst = &y->wu, want = F * H;
        else if (!strcmp(f, "wd")) dst = &y->wd, want = H * F;
    }
    if (!dst || n != want) return ORA_EINVAL;
    *dst = t;
    return ORA_OK;
}

static float *kslot(const ora_model *m, int l, int pos) {
    const ora_config *c = &m->c;
    return m->kcache + ((int64_t)l * c->max_seq + pos) * c->n_kv_heads * c->head_dim;
}
static float *vslot(const ora_model *m, int l, int pos) {
    const ora_config *c = &m->c;
    return m->vcache + ((int64_t)l * c->max_seq + pos) * c->n_kv_heads * c->head_dim;
}

/* Forward of ONE token at absolute position pos through the network with the
 * sublayers in `skip` bypassed (skip == NULL: the full target model).
 * Reads cache slots [0,pos) and writes slot pos in every non-skipped attention
 * sublayer.  logits: fp64 [vocab]. */
/* One token through the network at position pos.  reuse_kv = 0: the row's keys and values are
 * computed and written to cache slot pos before the row attends slots 0..pos.  reuse_kv = 1
 * (candidate evaluation): nothing is written; the row attends the keys and values that slots
 * 0..pos already hold. */
static int forward_row_general(ora_model *m, int32_t token, int pos, int slot, const int *extra, int n_extra,
                               int n_base, const uint8_t *skip, double *logits, int reuse_kv);

static int forward_row_impl(ora_model *m, int32_t token, int pos, const uint8_t *skip, double *logits, int reuse_kv) {
    return forward_row_general(m, token, pos, pos, NULL, 0, pos + 1, skip, logits, reuse_kv);
}

/* The general row: the token sits at sequence position `pos` (its rotary position), its keys and
 * values go to cache slot `slot`, and it attends slots 0 .. n_base-1 followed by the n_extra slots
 * listed in `extra` (in that order).  A plain row has slot = pos, n_base = pos + 1, no extra slots;
 * a row of a token tree attends the committed slots, then the slots of its ancestors in the block,
 * then its own. */
static int forward_row_general(ora_model *m, int32_t token, int pos, int slot, const int *extra, int n_extra,
                               int n_base, const uint8_t *skip, double *logits, int reuse_kv) {
    const ora_config *c = &m->c;
    if (token < 0 || token >= c->vocab) return ORA_EINVAL;
    if (pos < 0 || pos >= c->max_seq || slot < 0 || slot >= c->max_seq) return ORA_ECAPACITY;
    const int H = c->hidden, d = c->head_dim, nq = c->n_q_heads, nkv = c->n_kv_heads, F = c->ffn;
    const int n_att = n_base + n_extra;
    float *gk = NULL, *gv = NULL; /* gathered keys/values of the attended slots (tree rows only) */
    if (n_extra > 0) {
        gk = (float *)malloc(sizeof(float) * (size_t)n_att * (size_t)(nkv * d));
        gv = (float *)malloc(sizeof(float) * (size_t)n_att * (size_t)(nkv * d));
    }
    const int Q = nq * d, KV = nkv * d, group = nq / nkv;
    double *x = (double *)malloc(sizeof(double) * (size_t)H);
    double *xh = (double *)malloc(sizeof(double) * (size_t)H);
    double *q = (double *)malloc(sizeof(double) * (size_t)Q);
    double *k = (double *)malloc(sizeof(double) * (size_t)KV);
    double *v = (double *)malloc(sizeof(double) * (size_t)KV);
    double *att = (double *)malloc(sizeof(double) * (size_t)Q);
    double *tmp = (double *)malloc(sizeof(double) * (size_t)H);
    double *hg = (double *)malloc(sizeof(double) * (size_t)F);
    double *hu = (double *)malloc(sizeof(double) * (size_t)F);

    for (int i = 0; i < H; ++i) x[i] = tget(&m->embed, (int64_t)token * H + i);

    for (int l = 0; l < c->n_layers; ++l) {
        const ora_layer *y = &m->layers[l];
        if (!(skip && skip[2 * l])) {
            rmsnorm_t(x, &y->attn_norm, H, c->rms_eps, xh);
            matvec(m, &y->wq, Q, H, xh, q);
            for (int h = 0; h < nq; ++h) ora_rope(q + h * d, d, pos, c->rope_theta);
            if (!reuse_kv) {
                matvec(m, &y->wk, KV, H, xh, k);
                matvec(m, &y->wv, KV, H, xh, v);
                for (int h = 0; h < nkv; ++h) ora_rope(k + h * d, d, pos, c->rope_theta);
                float *ks = kslot(m, l, slot), *vs = vslot(m, l, slot);
                for (int i = 0; i < KV; ++i) {
                    ks[i] = round_kv(c, k[i]);
                    vs[i] = round_kv(c, v[i]);
                }
            }
            const float *kc = kslot(m, l, 0), *vc = vslot(m, l, 0);
            if (n_extra > 0) {
                for (int u = 0; u < n_att; ++u) {
                    const int src = u < n_base ? u : extra[u - n_base];
                    memcpy(gk + (size_t)u * KV, kslot(m, l, src), sizeof(float) * (size_t)KV);
                    memcpy(gv + (size_t)u * KV, vslot(m, l, src), sizeof(float) * (size_t)KV);
                }
                kc = gk;
                vc = gv;
            }
#pragma omp parallel for schedule(static) num_threads(m->threads)
            for (int h = 0; h < nq; ++h) {
                int g = h / group;
                ora_attend(q + h * d, kc + g * d, vc + g * d, KV, n_att, d, att + h * d);
            }
            matvec(m, &y->wo, H, Q, att, tmp);
            for (int i = 0; i < H; ++i) x[i] += tmp[i];
        }
        if (!(skip && skip[2 * l + 1])) {
            rmsnorm_t(x, &y->mlp_norm, H, c->rms_eps, xh);
            matvec(m, &y->wg, F, H, xh, hg);
            matvec(m, &y->wu, F, H, xh, hu);
            for (int i = 0; i < F; ++i) hg[i] = ora_swiglu(hg[i], hu[i]);
            matvec(m, &y->wd, H, F, hg, tmp);
            for (int i = 0; i < H; ++i) x[i] += tmp[i];
        }
    }
    rmsnorm_t(x, &m->final_norm, H, c->rms_eps, xh);
    matvec(m, &m->lm_head, c->vocab, H, xh, logits);

    free(x); free(xh); free(q); free(k); free(v); free(att); free(tmp); free(hg); free(hu);
    free(gk); free(gv);
    return ORA_OK;
}

int ora_forward_row(ora_model *m, int32_t token, int pos, const uint8_t *skip, double *logits) {
    return forward_row_impl(m, token, pos, skip, logits, 0);
}

/* Parallel candidate evaluation (Section 4.1.2).  window[0..gamma] are the tokens at positions
 * n - gamma .. n of the sequence decoded so far: window[0..gamma-1] are committed to the cache
 * (slots n - gamma .. n - 1 hold the target model's keys and values for them), window[gamma] is
 * the pending token.  The draft model with skipped set `skip` reads window[i-1] at position
 * n - gamma + i - 1, attends the target's cached keys and values of slots 0 .. n - gamma + i - 1
 * (Eq. 3: conditioned on x and y_<i; the target's cache is reused, nothing is written), and its
 * arg-max is the prediction y'_i of window[i], i = 1..gamma.  *n_match = number of i with
 * y'_i == window[i] (Eq. 4: matchness = *n_match / gamma).  The decoding state is not changed.
 * logits_out: NULL or fp64 [gamma][vocab]. */
int ora_eval_mask(ora_model *m, const uint8_t *skip, const int32_t *window, int gamma, int32_t *predicted,
                  int *n_match, double *logits_out) {
    if (!m || !skip || !window || gamma < 1) return ORA_EINVAL;
    if (m->pending < 0 || gamma > m->n) return ORA_ESTATE;
    const int V = m->c.vocab;
    double *lg = (double *)malloc(sizeof(double) * (size_t)V);
    int match = 0;
    for (int i = 1; i <= gamma; ++i) {
        int rc = forward_row_impl(m, window[i - 1], m->n - gamma + i - 1, skip, lg, 1);
        if (rc) {
            free(lg);
            return rc;
        }
        int32_t tok;
        ora_argmax_conf(lg, V, &tok, NULL);
        if (predicted) predicted[i - 1] = tok;
        if (logits_out) memcpy(logits_out + (size_t)(i - 1) * V, lg, sizeof(double) * (size_t)V);
        if (tok == window[i]) ++match;
    }
    free(lg);
    if (n_match) *n_match = match;
    return ORA_OK;
}

/* ---------------------------------------------------------------------------------------------
 * Optimisation phase: layer set suggestion by random search, candidate bookkeeping, termination
 * (Section 4.1, Appendix B.2).  Random numbers come from a counter-based generator that the GPU
 * library implements independently from the same definition:
 *     mix64(x): z = x + 0x9E3779B97F4A7C15; z = (z ^ z >> 30) * 0xBF58476D1CE4E5B9;
 *               z = (z ^ z >> 27) * 0x94D049BB133111EB; return z ^ z >> 31          (64-bit wrap)
 *     key(step) = mix64(mix64(seed ^ 0x53574946544F5054) + step)
 *     draw j of a step = mix64(key(step) + j)
 * The candidate of a step picks n_skip of the E eligible sublayers by a partial Fisher-Yates
 * shuffle of the eligible list (in index order): for j = 0 .. n_skip-1 swap entry j with entry
 * j + draw_j mod (E - j); the first n_skip entries are skipped.
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    int n_sublayers;        /* 2 * layers */
    double skip_ratio;      /* r: round(r * n_sublayers) sublayers are skipped */
    int max_steps;          /* S */
    int max_stale;          /* stop after this many steps without improvement */
    double stop_matchness;  /* stop when the best matchness exceeds this */
    uint64_t seed;
} ora_opt_config;

typedef struct ora_opt {
    ora_opt_config c;
    int *elig;              /* indices of the eligible sublayers, ascending */
    int n_elig, n_skip;
    uint8_t *best;
    double best_score;      /* -1 before the first evaluation */
    int step, stale, finished;
} ora_opt;

static uint64_t opt_mix64(uint64_t x) {
    uint64_t z = x + 0x9E3779B97F4A7C15ULL;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

int ora_opt_create(const ora_opt_config *c, const uint8_t *eligible, ora_opt **out) {
    if (!c || !out || c->n_sublayers < 1 || !(c->skip_ratio >= 0.0 && c->skip_ratio <= 1.0) || c->max_steps < 1 ||
        c->max_stale < 1)
        return ORA_EINVAL;
    ora_opt *o = (ora_opt *)calloc(1, sizeof(ora_opt));
    o->c = *c;
    o->elig = (int *)malloc(sizeof(int) * (size_t)c->n_sublayers);
    for (int i = 0; i < c->n_sublayers; ++i)
        if (!eligible || eligible[i]) o->elig[o->n_elig++] = i;
    o->n_skip = (int)floor(c->skip_ratio * (double)c->n_sublayers + 0.5);
    if (o->n_skip > o->n_elig) {
        free(o->elig);
        free(o);
        return ORA_EINVAL;
    }
    o->best = (uint8_t *)calloc((size_t)c->n_sublayers, 1);
    o->best_score = -1.0;
    *out = o;
    return ORA_OK;
}

void ora_opt_destroy(ora_opt *o) {
    if (!o) return;
    free(o->elig);
    free(o->best);
    free(o);
}

/* Uniform initial pattern (Section 4.1.1): the n_skip skipped sublayers are spread evenly over the
 * eligible ones: entry floor((j + 1/2) * E / n_skip) of the eligible list, j = 0 .. n_skip-1. */
void ora_opt_initial_mask(const ora_opt *o, uint8_t *mask) {
    memset(mask, 0, (size_t)o->c.n_sublayers);
    for (int j = 0; j < o->n_skip; ++j)
        mask[o->elig[(int)(((2 * (int64_t)j + 1) * o->n_elig) / (2 * (int64_t)o->n_skip))]] = 1;
}

/* Random-search candidate of optimisation step `step` (>= 1). */
void ora_opt_candidate(const ora_opt *o, int step, uint8_t *mask) {
    const int E = o->n_elig;
    int *perm = (int *)malloc(sizeof(int) * (size_t)(E > 0 ? E : 1));
    for (int i = 0; i < E; ++i) perm[i] = o->elig[i];
    const uint64_t key = opt_mix64(opt_mix64(o->c.seed ^ 0x53574946544F5054ULL) + (uint64_t)step);
    memset(mask, 0, (size_t)o->c.n_sublayers);
    for (int j = 0; j < o->n_skip; ++j) {
        const int pick = j + (int)(opt_mix64(key + (uint64_t)j) % (uint64_t)(E - j));
        const int t = perm[j];
        perm[j] = perm[pick];
        perm[pick] = t;
        mask[perm[j]] = 1;
    }
    free(perm);
}

/* One optimisation step before a decoding step: step 1 evaluates the uniform initial pattern,
 * every later step a random-search candidate, on the current context window (ora_eval_mask).  The
 * candidate replaces the retained one if its matchness is strictly higher.  finished: the step
 * limit is reached, or max_stale steps in a row brought no improvement, or the best matchness
 * exceeds stop_matchness.  Outputs (each may be NULL): the candidate and its matchness, the retained
 * set and its matchness, the finished flag.  ORA_ESTATE once finished. */
int ora_opt_step(ora_model *m, ora_opt *o, const int32_t *window, int gamma, uint8_t *cand_out, double *cand_score,
                 uint8_t *best_out, double *best_score, int *finished) {
    if (!m || !o || !window) return ORA_EINVAL;
    if (o->finished) return ORA_ESTATE;
    const int n = o->c.n_sublayers;
    if (n != 2 * m->c.n_layers) return ORA_EINVAL;
    uint8_t *cand = (uint8_t *)malloc((size_t)n);
    const int step = o->step + 1;
    if (step == 1)
        ora_opt_initial_mask(o, cand);
    else
        ora_opt_candidate(o, step, cand);
    int n_match = 0;
    int rc = ora_eval_mask(m, cand, window, gamma, NULL, &n_match, NULL);
    if (rc) {
        free(cand);
        return rc;
    }
    o->step = step;
    const double score = (double)n_match / (double)gamma;
    if (score > o->best_score) {
        memcpy(o->best, cand, (size_t)n);
        o->best_score = score;
        o->stale = 0;
    } else {
        o->stale++;
    }
    o->finished = o->step >= o->c.max_steps || o->stale >= o->c.max_stale || o->best_score > o->c.stop_matchness;
    if (cand_out) memcpy(cand_out, cand, (size_t)n);
    if (cand_score) *cand_score = score;
    if (best_out) memcpy(best_out, o->best, (size_t)n);
    if (best_score) *best_score = o->best_score;
    if (finished) *finished = o->finished;
    free(cand);
    return ORA_OK;
}

/* Brute force: logits of the LAST of n tokens from the full model, recomputed
 * from scratch, layer by layer over the whole sequence, with no cache and no
 * decoding state.  Keys and values pass through the same storage rounding. */
int ora_forward_nocache(ora_model *m, const int32_t *tokens, int n, double *logits) {
    const ora_config *c = &m->c;
    if (n <= 0) return ORA_EINVAL;
    const int H = c->hidden, d = c->head_dim, nq = c->n_q_heads, nkv = c->n_kv_heads, F = c->ffn;
    const int Q = nq * d, KV = nkv * d, group = nq / nkv;
    double *X = (double *)malloc(sizeof(double) * (size_t)n * H);
    double *xh = (double *)malloc(sizeof(double) * (size_t)H);
    double *Qm = (double *)malloc(sizeof(double) * (size_t)n * Q);
    float *Km = (float *)malloc(sizeof(float) * (size_t)n * KV);
    float *Vm = (float *)malloc(sizeof(float) * (size_t)n * KV);
    double *kv = (double *)malloc(sizeof(double) * (size_t)KV);
    double *att = (double *)malloc(sizeof(double) * (size_t)Q);
    double *tmp = (double *)malloc(sizeof(double) * (size_t)H);
    double *hg = (double *)malloc(sizeof(double) * (size_t)F);
    double *hu = (double *)malloc(sizeof(double) * (size_t)F);
    for (int t = 0; t < n; ++t) {
        if (tokens[t] < 0 || tokens[t] >= c->vocab) return ORA_EINVAL;
        for (int i = 0; i < H; ++i) X[(int64_t)t * H + i] = tget(&m->embed, (int64_t)tokens[t] * H + i);
    }
    for (int l = 0; l < c->n_layers; ++l) {
        const ora_layer *y = &m->layers[l];
        for (int t = 0; t < n; ++t) {
            rmsnorm_t(X + (int64_t)t * H, &y->attn_norm, H, c->rms_eps, xh);
            matvec(m, &y->wq, Q, H, xh, Qm + (int64_t)t * Q);
            for (int h = 0; h < nq; ++h) ora_rope(Qm + (int64_t)t * Q + h * d, d, t, c->rope_theta);
            matvec(m, &y->wk, KV, H, xh, kv);
            for (int h = 0; h < nkv; ++h) ora_rope(kv + h * d, d, t, c->rope_theta);
            for (int i = 0; i < KV; ++i) Km[(int64_t)t * KV + i] = round_kv(c, kv[i]);
            matvec(m, &y->wv, KV, H, xh, kv);
            for (int i = 0; i < KV; ++i) Vm[(int64_t)t * KV + i] = round_kv(c, kv[i]);
        }
        for (int t = 0; t < n; ++t) {
            for (int h = 0; h < nq; ++h) {
                int g = h / group;
                ora_attend(Qm + (int64_t)t * Q + h * d, Km + g * d, Vm + g * d, KV, t + 1, d, att + h * d);
            }
            matvec(m, &y->wo, H, Q, att, tmp);
            for (int i = 0; i < H; ++i) X[(int64_t)t * H + i] += tmp[i];
        }
        for (int t = 0; t < n; ++t) {
            rmsnorm_t(X + (int64_t)t * H, &y->mlp_norm, H, c->rms_eps, xh);
            matvec(m, &y->wg, F, H, xh, hg);
            matvec(m, &y->wu, F, H, xh, hu);
            for (int i = 0; i < F; ++i) hg[i] = ora_swiglu(hg[i], hu[i]);
            matvec(m, &y->wd, H, F, hg, tmp);
            for (int i = 0; i < H; ++i) X[(int64_t)t * H + i] += tmp[i];
        }
    }
    rmsnorm_t(X + (int64_t)(n - 1) * H, &m->final_norm, H, c->rms_eps, xh);
    matvec(m, &m->lm_head, c->vocab, H, xh, logits);
    free(X); free(xh); free(Qm); free(Km); free(Vm); free(kv); free(att); free(tmp); free(hg); free(hu);
    return ORA_OK;
}

/* ---------------------------------------------------------------- decoding steps */

int ora_reset(ora_model *m) {
    m->n = 0;
    m->pending = -1;
    m->k_draft = -1;
    m->k_verify = -1;
    m->tree_levels = -1;
    m->k_sampled = -1;
    m->n_draft_passes = m->n_verify_passes = m->n_accepted = m->n_emitted = 0;
    return ORA_OK;
}

/* Prefill: the full model over the prompt at positions 0..P-1; the arg-max of
 * the last row is the first new token (becomes the pending token). */
int ora_prefill(ora_model *m, const int32_t *prompt, int P, int32_t *first_token, double *last_logits) {
    if (!m || !prompt || P <= 0) return ORA_EINVAL;
    if (P >= m->c.max_seq) return ORA_ECAPACITY;
    ora_reset(m);
    double *lg = (double *)malloc(sizeof(double) * (size_t)m->c.vocab);
    for (int t = 0; t < P; ++t) {
        int rc = ora_forward_row(m, prompt[t], t, NULL, lg);
        if (rc) {
            free(lg);
            return rc;
        }
    }
    int32_t tok;
    ora_argmax_conf(lg, m->c.vocab, &tok, NULL);
    if (last_logits) memcpy(last_logits, lg, sizeof(double) * (size_t)m->c.vocab);
    free(lg);
    m->n = P;
    m->pending = tok;
    m->n_emitted = 1;
    if (first_token) *first_token = tok;
    return ORA_OK;
}

/* Drafting (Section 4.2, Eq. 5 and strategy 1): starting from the pending
 * token at position n, run the draft model autoregressively; draft token j is
 * the arg-max, its confidence the top-1 probability; stop after the token
 * whose confidence is below the threshold (that token is kept) or after max_k
 * tokens.  Draft keys/values go to slots n, n+1, ... of the non-skipped
 * attention sublayers and are overwritten by the next verify. */
int ora_draft_step(ora_model *m, const uint8_t *skip, int max_k, double conf_threshold, int32_t *draft_tokens,
                   double *draft_conf, int *k_out) {
    if (!m || !skip || max_k < 0 || max_k > ORA_MAX_BLOCK) return ORA_EINVAL;
    if (m->pending < 0) return ORA_ESTATE;
    if (m->n + max_k + 1 > m->c.max_seq) return ORA_ECAPACITY;
    double *lg = (double *)malloc(sizeof(double) * (size_t)m->c.vocab);
    int32_t prev = m->pending;
    int k = 0;
    for (int j = 1; j <= max_k; ++j) {
        int rc = ora_forward_row(m, prev, m->n + j - 1, skip, lg);
        if (rc) {
            free(lg);
            return rc;
        }
        int32_t tok;
        double p;
        ora_argmax_conf(lg, m->c.vocab, &tok, &p);
        m->n_draft_passes++;
        m->draft[k] = tok;
        if (draft_tokens) draft_tokens[k] = tok;
        if (draft_conf) draft_conf[k] = p;
        ++k;
        prev = tok;
        if (p < conf_threshold) break;
    }
    free(lg);
    m->k_draft = k;
    m->k_sampled = -1;
    if (k_out) *k_out = k;
    return ORA_OK;
}

/* Verification: the full model over rows [tokens[0..k]] at positions n..n+k;
 * row i sees slots 0..n+i.  Target keys/values overwrite slots n..n+k in every
 * layer.  target_tokens[i] = arg-max of row i.  logits_out: NULL or fp64 [k+1][vocab]. */
int ora_verify(ora_model *m, const int32_t *tokens, int k, int32_t *target_tokens, double *logits_out) {
    if (!m || !tokens || k < 0 || k > ORA_MAX_BLOCK) return ORA_EINVAL;
    if (m->pending < 0) return ORA_ESTATE;
    if (m->n + k + 1 > m->c.max_seq) return ORA_ECAPACITY;
    double *lg = (double *)malloc(sizeof(double) * (size_t)m->c.vocab);
    for (int i = 0; i <= k; ++i) {
        int rc = ora_forward_row(m, tokens[i], m->n + i, NULL, lg);
        if (rc) {
            free(lg);
            return rc;
        }
        int32_t tok;
        ora_argmax_conf(lg, m->c.vocab, &tok, NULL);
        m->vtokens[i] = tokens[i];
        m->target[i] = tok;
        if (target_tokens) target_tokens[i] = tok;
        if (logits_out) memcpy(logits_out + (int64_t)i * m->c.vocab, lg, sizeof(double) * (size_t)m->c.vocab);
    }
    free(lg);
    m->k_verify = k;
    m->tree_levels = -1;
    m->n_verify_passes++;
    return ORA_OK;
}

/* Acceptance and roll-back: m = longest prefix of the verified draft tokens
 * that equals the target's greedy tokens; emit those m tokens and the target's
 * own next token g_m; cache length becomes n + m + 1; g_m is the new pending token. */
int ora_accept(ora_model *m, int32_t *emitted, int *n_emitted) {
    if (!m) return ORA_EINVAL;
    if (m->k_verify < 0) return ORA_ESTATE;
    int k = m->k_verify;
    int acc = ora_match_prefix(m->vtokens + 1, m->target, k);
    for (int i = 0; i < acc; ++i)
        if (emitted) emitted[i] = m->vtokens[1 + i];
    if (emitted) emitted[acc] = m->target[acc];
    if (n_emitted) *n_emitted = acc + 1;
    m->n += acc + 1;
    m->pending = m->target[acc];
    m->n_accepted += acc;
    m->n_emitted += acc + 1;
    m->k_verify = -1;
    m->k_draft = -1;
    return ORA_OK;
}

/* ---------------------------------------------------------------------------------------------
 * Dynamic verification (Section 4.2, strategy 2)
 * ------------------------------------------------------------------------------------------- */
/* Candidates per draft position from its confidence p (the paper's four bands). */
int ora_topk_width(double p) {
    if (p <= 0.5) return 10;
    if (p <= 0.8) return 5;
    if (p <= 0.95) return 3;
    return 1;
}

/* The k largest logits (compared in fp32, as the arg-max is), largest first; equal values in
 * index order.  tokens[0] is the arg-max. */
void ora_topk(const double *logits, int n, int k, int32_t *tokens) {
    for (int j = 0; j < k; ++j) {
        int best = -1;
        float bv = 0.f;
        for (int i = 0; i < n; ++i) {
            int taken = 0;
            for (int t = 0; t < j; ++t) taken |= tokens[t] == i;
            if (taken) continue;
            float v = (float)logits[i];
            if (best < 0 || v > bv) {
                bv = v;
                best = i;
            }
        }
        tokens[j] = best;
    }
}

/* Drafting as in ora_draft_step, keeping for every draft position j its top candidates
 * tokens[j][0..width[j]) (tokens[j][0] is the draft token the next position continues from) with
 * width[j] = min(ora_topk_width(p_j), max_width, rows left), where a block holds at most
 * min(ORA_TREE_ROWS, max_seq - n) rows (the pending token and all candidates; every row needs a cache
 * slot of its own); drafting also stops when no row is left.  tokens: [max_k][ORA_TOPK]. */
int ora_draft_step_topk(ora_model *m, const uint8_t *skip, int max_k, double conf_threshold, int max_width,
                        int32_t *tokens, double *draft_conf, int *width, int *k_out) {
    if (!m || !skip || !tokens || !width || max_k < 0 || max_k > ORA_TREE_ROWS - 1 || max_width < 1) return ORA_EINVAL;
    if (m->pending < 0) return ORA_ESTATE;
    const int cap_rows = m->c.max_seq - m->n < ORA_TREE_ROWS ? m->c.max_seq - m->n : ORA_TREE_ROWS;
    if (cap_rows < 1) return ORA_ECAPACITY;
    double *lg = (double *)malloc(sizeof(double) * (size_t)m->c.vocab);
    int32_t prev = m->pending;
    int k = 0, rows = 1;
    for (int j = 1; j <= max_k && rows < cap_rows; ++j) {
        int rc = ora_forward_row(m, prev, m->n + j - 1, skip, lg);
        if (rc) {
            free(lg);
            return rc;
        }
        int32_t tok;
        double p;
        ora_argmax_conf(lg, m->c.vocab, &tok, &p);
        m->n_draft_passes++;
        int w = ora_topk_width(p);
        if (w > max_width) w = max_width;
        if (w > cap_rows - rows) w = cap_rows - rows;
        if (w > m->c.vocab) w = m->c.vocab;
        ora_topk(lg, m->c.vocab, w, tokens + (size_t)k * ORA_TOPK);
        width[k] = w;
        if (draft_conf) draft_conf[k] = p;
        m->draft[k] = tok;
        rows += w;
        ++k;
        prev = tok;
        if (p < conf_threshold) break;
    }
    free(lg);
    m->k_draft = k;
    m->k_sampled = -1;
    if (k_out) *k_out = k;
    return ORA_OK;
}

/* Verification of a token tree in one block.  Row 0 is the pending token; level j = 1..levels has
 * width[j-1] rows, the candidates of draft position j, the first of them the draft token itself
 * (the "spine").  tokens: the rows in order (row 0, level 1, level 2, ...).  A row of level j sits
 * at sequence position n + j; its keys/values go to cache slot n + row; it attends the committed
 * slots 0..n-1, row 0, the spine rows of levels 1..j-1, and itself.  target_tokens[row] = arg-max
 * of the row = the target model's next token after the path that ends in that row. */
int ora_verify_tree(ora_model *m, const int32_t *tokens, const int *width, int levels, int32_t *target_tokens,
                    double *logits_out) {
    if (!m || !tokens || levels < 0 || levels > ORA_TREE_ROWS - 1 || (levels > 0 && !width)) return ORA_EINVAL;
    if (m->pending < 0) return ORA_ESTATE;
    int rows = 1;
    for (int j = 0; j < levels; ++j) {
        if (width[j] < 1 || width[j] > ORA_TOPK) return ORA_EINVAL;
        rows += width[j];
    }
    if (rows > ORA_TREE_ROWS) return ORA_EINVAL;
    if (m->n + rows > m->c.max_seq) return ORA_ECAPACITY;
    const int V = m->c.vocab, n = m->n;
    double *lg = (double *)malloc(sizeof(double) * (size_t)V);
    int extra[ORA_TREE_ROWS + 1];
    int n_spine = 0; /* extra[0..n_spine) = slots of row 0 and of the spine rows of the levels done */
    int row = 0;
    for (int j = 0; j <= levels; ++j) {
        const int w = j == 0 ? 1 : width[j - 1];
        const int first = row;
        for (int i = 0; i < w; ++i, ++row) {
            extra[n_spine] = n + row; /* itself, after its ancestors */
            int rc = forward_row_general(m, tokens[row], n + j, n + row, extra, n_spine + 1, n, NULL, lg, 0);
            if (rc) {
                free(lg);
                return rc;
            }
            int32_t tok;
            ora_argmax_conf(lg, V, &tok, NULL);
            m->tree_tokens[row] = tokens[row];
            m->tree_target[row] = tok;
            if (target_tokens) target_tokens[row] = tok;
            if (logits_out) memcpy(logits_out + (int64_t)row * V, lg, sizeof(double) * (size_t)V);
        }
        extra[n_spine++] = n + first; /* the first row of the level is the ancestor of the next levels */
    }
    free(lg);
    m->tree_levels = levels;
    for (int j = 0; j < levels; ++j) m->tree_width[j] = width[j];
    m->k_verify = -1;
    m->n_verify_passes++;
    return ORA_OK;
}

/* Acceptance on the tree: starting from the target's token after the pending token, a level is
 * accepted if one of its candidates equals the target's token for the path so far; the path goes on
 * only through the spine (the other candidates were not extended by the draft model).  Emits the
 * accepted candidates and the target's own next token, moves the keys/values of the accepted rows to
 * slots n+1 .. n+m (row 0 already sits in slot n), and sets cache length n + m + 1. */
int ora_accept_tree(ora_model *m, int32_t *emitted, int *n_emitted) {
    if (!m) return ORA_EINVAL;
    if (m->tree_levels < 0) return ORA_ESTATE;
    const ora_config *c = &m->c;
    const int KV = c->n_kv_heads * c->head_dim;
    int32_t cur = m->tree_target[0];
    int acc = 0, start = 1;
    for (int j = 1; j <= m->tree_levels; ++j) {
        const int w = m->tree_width[j - 1];
        int hit = -1;
        for (int i = 0; i < w; ++i)
            if (m->tree_tokens[start + i] == cur) {
                hit = i;
                break;
            }
        if (hit < 0) break;
        const int row = start + hit;
        if (emitted) emitted[acc] = cur;
        ++acc;
        if (row != acc) /* accepted row's keys/values to slot n + acc */
            for (int l = 0; l < c->n_layers; ++l) {
                memcpy(kslot(m, l, m->n + acc), kslot(m, l, m->n + row), sizeof(float) * (size_t)KV);
                memcpy(vslot(m, l, m->n + acc), vslot(m, l, m->n + row), sizeof(float) * (size_t)KV);
            }
        cur = m->tree_target[row];
        if (hit != 0) break; /* a candidate beside the spine has no children */
        start += w;
    }
    if (emitted) emitted[acc] = cur;
    if (n_emitted) *n_emitted = acc + 1;
    m->n += acc + 1;
    m->pending = cur;
    m->n_accepted += acc;
    m->n_emitted += acc + 1;
    m->tree_levels = -1;
    m->k_draft = -1;
    return ORA_OK;
}

/* ---------------------------------------------------------------------------------------------
 * Speculative sampling (Section 5.1 and Appendix B.2: acceptance by speculative sampling,
 * temperature 0.6 and top-p 0.95 for the sampled runs)
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    double p;
    int i;
} prob_idx;
static int by_prob_desc(const void *a, const void *b) {
    const prob_idx *x = (const prob_idx *)a, *y = (const prob_idx *)b;
    if (x->p != y->p) return x->p > y->p ? -1 : 1;
    return x->i - y->i;
}

/* The distribution tokens are drawn from: softmax(logits / temperature), restricted to the nucleus
 * and renormalised.  Nucleus: walk the tokens from the most to the least probable and stop at the
 * first one with which the probabilities add up to top_p or more; every token as probable as that
 * last one belongs to it too.  top_p >= 1 keeps everything.
 * margin (may be NULL): how far the cut was from falling elsewhere: the smaller of (sum with the
 * cut's ties - top_p), (top_p - sum before the cut's probability value) and the relative gap to
 * the next smaller probability. */
void ora_warp(const double *logits, int n, double temperature, double top_p, double *probs, double *margin) {
    double mx = logits[0];
    for (int i = 1; i < n; ++i)
        if (logits[i] > mx) mx = logits[i];
    double z = 0.0;
    for (int i = 0; i < n; ++i) {
        probs[i] = exp((logits[i] - mx) / temperature);
        z += probs[i];
    }
    for (int i = 0; i < n; ++i) probs[i] /= z;
    if (margin) *margin = 1.0;
    if (top_p >= 1.0) return;
    prob_idx *o = (prob_idx *)malloc(sizeof(prob_idx) * (size_t)n);
    for (int i = 0; i < n; ++i) {
        o[i].p = probs[i];
        o[i].i = i;
    }
    qsort(o, (size_t)n, sizeof(prob_idx), by_prob_desc);
    double cum = 0.0;
    int j = 0;
    for (; j < n; ++j) {
        cum += o[j].p;
        if (cum >= top_p) break;
    }
    if (j == n) j = n - 1; /* rounding left the total a hair below top_p: everything stays */
    const double cut = o[j].p;
    double before = 0.0, with_ties = 0.0;
    int last = j;
    for (int t = 0; t < n; ++t) {
        if (o[t].p > cut) before += o[t].p;
        if (o[t].p >= cut) {
            with_ties += o[t].p;
            last = t;
        }
    }
    if (margin) {
        double mg = with_ties - top_p;
        if (top_p - before < mg) mg = top_p - before;
        if (last + 1 < n && (cut - o[last + 1].p) / cut < mg) mg = (cut - o[last + 1].p) / cut;
        *margin = mg;
    }
    for (int i = 0; i < n; ++i)
        if (probs[i] < cut) probs[i] = 0.0;
    for (int i = 0; i < n; ++i) probs[i] /= with_ties;
    free(o);
}

/* Inverse-CDF draw in token-id order from non-negative weights w (need not be normalised):
 * the first token j with w_0 + .. + w_j > u * total, u in [0, 1).  margin (may be NULL): distance
 * of u from the two ends of the chosen token's interval, on the normalised scale. */
int ora_sample(const double *w, int n, double u, double *margin) {
    double total = 0.0;
    for (int i = 0; i < n; ++i) total += w[i];
    double c = 0.0;
    int last = -1;
    for (int j = 0; j < n; ++j) {
        if (w[j] <= 0.0) continue;
        last = j;
        const double c0 = c;
        c += w[j];
        if (c > u * total) {
            if (margin) {
                double a = c / total - u, b = u - c0 / total;
                *margin = a < b ? a : b;
            }
            return j;
        }
    }
    if (margin) *margin = 0.0;
    return last; /* u * total reached the total through rounding */
}

/* One acceptance decision: draft token x drawn from q is kept iff u < min(1, p[x] / q[x]). */
int ora_spec_keep(double p_x, double q_x, double u, double *margin) {
    if (margin) *margin = fabs(p_x - u * q_x) / (q_x > 0.0 ? q_x : 1.0);
    return u * q_x < p_x;
}

/* The replacement token after a rejection: drawn from max(0, p - q) renormalised (from p itself
 * if p == q everywhere). */
int ora_spec_resample(const double *p, const double *q, int n, double u, double *margin) {
    double *r = (double *)malloc(sizeof(double) * (size_t)n);
    double tot = 0.0;
    for (int i = 0; i < n; ++i) {
        r[i] = p[i] > q[i] ? p[i] - q[i] : 0.0;
        tot += r[i];
    }
    int tok = tot > 0.0 ? ora_sample(r, n, u, margin) : ora_sample(p, n, u, margin);
    free(r);
    return tok;
}

/* Test helper: the first token a speculative step with one draft token emits, given target and
 * draft distributions p, q over n tokens and the three uniforms (draw, acceptance, replacement);
 * out[i] for triples u[3i..3i+2]. */
void ora_spec_first_token_batch(const double *p, const double *q, int n, const double *u, int64_t count, int32_t *out) {
    for (int64_t i = 0; i < count; ++i) {
        const int x = ora_sample(q, n, u[3 * i], NULL);
        out[i] = ora_spec_keep(p[x], q[x], u[3 * i + 1], NULL) ? x : ora_spec_resample(p, q, n, u[3 * i + 2], NULL);
    }
}

/* Prefill whose first token is drawn from the warped distribution of the last prompt row. */
int ora_prefill_sample(ora_model *m, const int32_t *prompt, int P, double temperature, double top_p, double u,
                       int32_t *first_token, double *min_margin) {
    if (!m || temperature <= 0.0 || top_p <= 0.0 || u < 0.0 || u >= 1.0) return ORA_EINVAL;
    const int V = m->c.vocab;
    double *lg = (double *)malloc(sizeof(double) * (size_t)V * 2), *pr = lg + V;
    int32_t greedy;
    int rc = ora_prefill(m, prompt, P, &greedy, lg);
    if (rc) {
        free(lg);
        return rc;
    }
    double m1, m2;
    ora_warp(lg, V, temperature, top_p, pr, &m1);
    const int tok = ora_sample(pr, V, u, &m2);
    free(lg);
    m->pending = tok;
    if (first_token) *first_token = tok;
    if (min_margin) *min_margin = m1 < m2 ? m1 : m2;
    return ORA_OK;
}

/* Drafting with sampling: as ora_draft_step, but draft token j is drawn with u[j-1] from the warped
 * distribution q_j of the draft model's logits, which is kept for the acceptance test.  The
 * confidence that ends drafting early stays the top-1 probability of the plain softmax. */
int ora_draft_step_sample(ora_model *m, const uint8_t *skip, int max_k, double conf_threshold, double temperature,
                          double top_p, const double *u, int32_t *draft_tokens, double *draft_conf, int *k_out,
                          double *min_margin) {
    if (!m || !skip || max_k < 0 || max_k > ORA_TREE_ROWS - 1 || temperature <= 0.0 || top_p <= 0.0) return ORA_EINVAL;
    if (max_k > 0 && !u) return ORA_EINVAL;
    if (m->pending < 0) return ORA_ESTATE;
    if (m->n + max_k + 1 > m->c.max_seq) return ORA_ECAPACITY;
    const int V = m->c.vocab;
    if (!m->qdist) m->qdist = (double *)malloc(sizeof(double) * (size_t)V * ORA_TREE_ROWS);
    double *lg = (double *)malloc(sizeof(double) * (size_t)V);
    int32_t prev = m->pending;
    int k = 0;
    double mm = 1.0;
    for (int j = 1; j <= max_k; ++j) {
        if (u[j - 1] < 0.0 || u[j - 1] >= 1.0) {
            free(lg);
            return ORA_EINVAL;
        }
        int rc = ora_forward_row(m, prev, m->n + j - 1, skip, lg);
        if (rc) {
            free(lg);
            return rc;
        }
        int32_t top;
        double p, m1, m2;
        ora_argmax_conf(lg, V, &top, &p);
        double *q = m->qdist + (size_t)k * V;
        ora_warp(lg, V, temperature, top_p, q, &m1);
        const int tok = ora_sample(q, V, u[j - 1], &m2);
        if (m1 < mm) mm = m1;
        if (m2 < mm) mm = m2;
        m->n_draft_passes++;
        m->draft[k] = tok;
        if (draft_tokens) draft_tokens[k] = tok;
        if (draft_conf) draft_conf[k] = p;
        ++k;
        prev = tok;
        if (p < conf_threshold) break;
    }
    free(lg);
    m->k_draft = k;
    m->k_sampled = k;
    if (k_out) *k_out = k;
    if (min_margin) *min_margin = mm;
    return ORA_OK;
}

/* Verification and acceptance with sampling: the target model over [pending, x_1..x_k] (the tokens
 * of the last ora_draft_step_sample); p_i = warped distribution of row i-1.  x_i is kept iff
 * u_accept[i-1] < min(1, p_i(x_i) / q_i(x_i)); the first rejected position gets a token drawn with
 * u_final from max(0, p_i - q_i) renormalised and ends the step; if all k are kept, one more token is
 * drawn with u_final from p_{k+1}.  State afterwards as after ora_accept.  k = 0: one step of plain
 * sampling.  probs_out: NULL or [k+1][vocab], the target's warped distributions. */
int ora_verify_sample(ora_model *m, const int32_t *tokens, int k, double temperature, double top_p, const double *u_accept,
                      double u_final, int32_t *emitted, int *n_emitted, double *probs_out, double *min_margin) {
    if (!m || !tokens || k < 0 || k > ORA_TREE_ROWS - 1 || temperature <= 0.0 || top_p <= 0.0) return ORA_EINVAL;
    if (u_final < 0.0 || u_final >= 1.0 || (k > 0 && !u_accept)) return ORA_EINVAL;
    if (m->pending < 0) return ORA_ESTATE;
    if (tokens[0] != m->pending) return ORA_EINVAL;
    if (k > 0 && (m->k_sampled < k || !m->qdist)) return ORA_ESTATE;
    for (int i = 0; i < k; ++i)
        if (tokens[1 + i] != m->draft[i]) return ORA_EINVAL;
    const int V = m->c.vocab;
    double *lgs = (double *)malloc(sizeof(double) * (size_t)V * (size_t)(k + 2));
    double *pr = lgs + (size_t)V * (size_t)(k + 1);
    int rc = ora_verify(m, tokens, k, NULL, lgs);
    if (rc) {
        free(lgs);
        return rc;
    }
    double mm = 1.0, mg;
    int acc = 0;
    int32_t last = -1;
    for (int i = 0; i <= k; ++i) {
        ora_warp(lgs + (size_t)i * V, V, temperature, top_p, pr, &mg);
        if (mg < mm) mm = mg;
        if (probs_out) memcpy(probs_out + (size_t)i * V, pr, sizeof(double) * (size_t)V);
        if (i == k) {
            last = ora_sample(pr, V, u_final, &mg);
            if (mg < mm) mm = mg;
            break;
        }
        const double *q = m->qdist + (size_t)i * V;
        const int x = tokens[1 + i];
        const int keep = ora_spec_keep(pr[x], q[x], u_accept[i], &mg);
        if (mg < mm) mm = mg;
        if (!keep) {
            last = ora_spec_resample(pr, q, V, u_final, &mg);
            if (mg < mm) mm = mg;
            break;
        }
        if (emitted) emitted[acc] = x;
        ++acc;
    }
    free(lgs);
    if (emitted) emitted[acc] = last;
    if (n_emitted) *n_emitted = acc + 1;
    m->n += acc + 1;
    m->pending = last;
    m->n_accepted += acc;
    m->n_emitted += acc + 1;
    m->k_verify = -1;
    m->k_draft = -1;
    m->k_sampled = -1;
    if (min_margin) *min_margin = mm;
    return ORA_OK;
}

/* Sets the cache length to new_len <= current and the pending token; no data is touched. */
int ora_rollback(ora_model *m, int new_len, int32_t pending) {
    if (!m || new_len < 0 || new_len > m->n || pending < 0 || pending >= m->c.vocab) return ORA_EINVAL;
    if (m->pending < 0) return ORA_ESTATE;
    m->n = new_len;
    m->pending = pending;
    m->k_draft = m->k_verify = m->k_sampled = -1;
    m->tree_levels = -1;
    return ORA_OK;
}

int ora_cache_len(const ora_model *m) { return m->n; }
int ora_pending(const ora_model *m) { return m->pending; }

/* counters: [draft passes, verify passes, accepted draft tokens, emitted tokens] */
void ora_get_stats(const ora_model *m, int64_t out[4]) {
    out[0] = m->n_draft_passes;
    out[1] = m->n_verify_passes;
    out[2] = m->n_accepted;
    out[3] = m->n_emitted;
}

/* Test hook: NaN-fill every cache slot at or beyond the cache length. */
void ora_poison_kv(ora_model *m) {
    const ora_config *c = &m->c;
    int64_t w = (int64_t)c->n_kv_heads * c->head_dim;
    for (int l = 0; l < c->n_layers; ++l)
        for (int p = m->n; p < c->max_seq; ++p)
            for (int64_t i = 0; i < w; ++i) kslot(m, l, p)[i] = vslot(m, l, p)[i] = NAN;
}

/* Test access to the cache: copy slot `pos` of layer l (keys then values, fp32). */
void ora_read_kv(const ora_model *m, int l, int pos, float *k_out, float *v_out) {
    int64_t w = (int64_t)m->c.n_kv_heads * m->c.head_dim;
    memcpy(k_out, kslot(m, l, pos), sizeof(float) * (size_t)w);
    memcpy(v_out, vslot(m, l, pos), sizeof(float) * (size_t)w);
}
