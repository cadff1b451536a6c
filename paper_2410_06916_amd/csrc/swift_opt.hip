// Host logic of the optimisation phase on top of swift_eval_mask: layer set suggestion by random
// search under a fixed skip ratio, the uniform initial pattern, retention of the best candidate and
// the termination rules (paper Sections 4.1.1 and 4.1.2, Eq. 2; Appendix B.2).  No device code here:
// the one expensive part of a step, the candidate's block pass over the context window, is
// swift_eval_mask.
#include <stdint.h>
#include <string.h>

#include <cmath>
#include <vector>

#include "../../include/swift.h"

struct swift_opt {
    swift_opt_config c;
    std::vector<int> eligible;  // sublayers that may be skipped, ascending
    int n_skip;
    std::vector<uint8_t> best;
    double best_score;  // -1: nothing evaluated yet
    int step, stale;
    bool finished;
    swift_suggest_fn suggest;  // optional: replaces random search every `interval` steps
    void *suggest_user;
    int suggest_interval;
};

namespace {

// splitmix64 output function applied to x + its increment
uint64_t mix64(uint64_t x) {
    uint64_t z = x + 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

void uniform_pattern(const swift_opt *o, uint8_t *mask) {
    memset(mask, 0, (size_t)o->c.n_sublayers);
    const int64_t E = (int64_t)o->eligible.size();
    for (int64_t j = 0; j < o->n_skip; ++j) mask[o->eligible[(size_t)(((2 * j + 1) * E) / (2 * (int64_t)o->n_skip))]] = 1;
}

// n_skip of the eligible sublayers by a partial Fisher-Yates shuffle driven by the counter-based
// stream of this (seed, step)
void random_candidate(const swift_opt *o, int step, uint8_t *mask) {
    std::vector<int> perm(o->eligible);
    const uint64_t key = mix64(mix64(o->c.seed ^ 0x53574946544F5054ull) + (uint64_t)step);
    memset(mask, 0, (size_t)o->c.n_sublayers);
    const size_t E = perm.size();
    for (size_t j = 0; j < (size_t)o->n_skip; ++j) {
        const size_t pick = j + (size_t)(mix64(key + (uint64_t)j) % (uint64_t)(E - j));
        std::swap(perm[j], perm[pick]);
        mask[perm[j]] = 1;
    }
}

}  // namespace

extern "C" int swift_opt_create(const swift_opt_config *cfg, const uint8_t *eligible, swift_opt **out) {
    if (!cfg || !out) return SWIFT_EINVAL;
    *out = nullptr;
    if (cfg->n_sublayers < 1 || !(cfg->skip_ratio >= 0.0 && cfg->skip_ratio <= 1.0) || cfg->max_steps < 1 ||
        cfg->max_stale < 1)
        return SWIFT_EINVAL;
    swift_opt *o = new swift_opt();
    o->c = *cfg;
    for (int i = 0; i < cfg->n_sublayers; ++i)
        if (!eligible || eligible[i]) o->eligible.push_back(i);
    o->n_skip = (int)std::floor(cfg->skip_ratio * (double)cfg->n_sublayers + 0.5);
    if (o->n_skip > (int)o->eligible.size()) {
        delete o;
        return SWIFT_EINVAL;
    }
    o->best.assign((size_t)cfg->n_sublayers, 0);
    o->best_score = -1.0;
    o->step = o->stale = 0;
    o->finished = false;
    o->suggest = nullptr;
    o->suggest_user = nullptr;
    o->suggest_interval = 0;
    *out = o;
    return SWIFT_OK;
}

extern "C" int swift_opt_destroy(swift_opt *o) {
    if (!o) return SWIFT_EINVAL;
    delete o;
    return SWIFT_OK;
}

extern "C" int swift_opt_initial_mask(const swift_opt *o, uint8_t *mask) {
    if (!o || !mask) return SWIFT_EINVAL;
    uniform_pattern(o, mask);
    return SWIFT_OK;
}

extern "C" int swift_opt_candidate(const swift_opt *o, int step, uint8_t *mask) {
    if (!o || !mask || step < 1) return SWIFT_EINVAL;
    random_candidate(o, step, mask);
    return SWIFT_OK;
}

extern "C" int swift_opt_set_suggester(swift_opt *o, swift_suggest_fn fn, void *user, int interval) {
    if (!o || (fn && interval < 1)) return SWIFT_EINVAL;
    o->suggest = fn;
    o->suggest_user = user;
    o->suggest_interval = fn ? interval : 0;
    return SWIFT_OK;
}

extern "C" int swift_opt_step(swift_ctx *ctx, swift_opt *o, const int32_t *window, int gamma, uint8_t *candidate,
                              double *candidate_matchness, uint8_t *best_mask, double *best_matchness, int *finished) {
    if (!ctx || !o || !window) return SWIFT_EINVAL;
    if (o->finished) return SWIFT_ESTATE;
    const int n = o->c.n_sublayers;
    // the candidate is indexed as a skip mask of the context's model: one entry per sublayer
    swift_model_config mc;
    if (swift_get_config(ctx, &mc) != SWIFT_OK || n != 2 * mc.n_layers) return SWIFT_EINVAL;
    std::vector<uint8_t> cand((size_t)n, 0);
    const int step = o->step + 1;
    bool have = false;
    if (step == 1) {
        uniform_pattern(o, cand.data());
        have = true;
    } else if (o->suggest && step % o->suggest_interval == 0) {
        // an external suggester (e.g. Bayesian optimisation over the scores so far) may take this step
        have = o->suggest(o->suggest_user, step, o->best.data(), o->best_score, n, cand.data()) == 0;
    }
    if (!have) random_candidate(o, step, cand.data());
    int n_match = 0;
    const int rc = swift_eval_mask(ctx, cand.data(), window, gamma, nullptr, &n_match);
    if (rc != SWIFT_OK) return rc;
    o->step = step;
    const double score = (double)n_match / (double)gamma;
    if (score > o->best_score) {
        o->best = cand;
        o->best_score = score;
        o->stale = 0;
    } else {
        o->stale++;
    }
    o->finished = o->step >= o->c.max_steps || o->stale >= o->c.max_stale || o->best_score > o->c.stop_matchness;
    if (candidate) memcpy(candidate, cand.data(), (size_t)n);
    if (candidate_matchness) *candidate_matchness = score;
    if (best_mask) memcpy(best_mask, o->best.data(), (size_t)n);
    if (best_matchness) *best_matchness = o->best_score;
    if (finished) *finished = o->finished ? 1 : 0;
    return SWIFT_OK;
}
