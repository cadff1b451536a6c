"""GPU parity of speculative sampling (Section 5.1, Appendix B.2) against the CPU oracle: with the same
uniforms both sides draw the same tokens, keep the same drafts and replace the same ones, step by step,
wherever the oracle reports that no decision was closer to falling the other way than the two sides'
arithmetic can differ (fp64 against fp32); the target distributions agree to the logits' tolerance; and
what a step emits is distributed as the target model's own samples."""
import numpy as np
import pytest

import synthetic_inputs as si
from tests import helpers as hp

pytestmark = pytest.mark.gpu

# how far a decision must be from its boundary for the two sides to be held to the same outcome, and the
# tolerance on the target probabilities (they inherit the logits' tolerance divided by the temperature)
MARGIN = {"fp32": 1e-4, "bf16": 5e-4}
PROB_TOL = {"fp32": 2e-4, "bf16": 1e-2}

_CASES = {
    "small-gqa": (hp.SMALL_GQA, 96, 12),
    "small-gqa-bf16": (hp.SMALL_GQA_BF16, 96, 12),
    "small-gqa-bf16-long-cache": (hp.SMALL_GQA_BF16, 1700, 70),
    "big-vocab": (si.ModelShape("big-vocab", 1, 64, 2, 1, 32, 96, 33002, "bf16", 1e-5), 80, 9),
}


def _pair(oracle_lib, shape, weights, max_seq):
    import paper_2410_06916_amd as P
    o = oracle_lib.Oracle(shape, max_seq, threads=4)
    o.set_weights(weights)
    g = P.SwiftModel(shape, max_seq)
    g.load_weights(weights)
    return o, g


def _lockstep(o, g, shape, prompt, n_new, mask, max_k, eps, T, top_p, u0, U):
    """Runs both sides step by step with the same uniforms.  Returns (steps compared, steps run, kept,
    replaced); stops at the first step where a low-margin decision fell differently."""
    thr, ptol = MARGIN[shape.dtype], PROB_TOL[shape.dtype]
    to, mg = o.prefill_sample(prompt, T, top_p, u0)
    tg = g.prefill_sample(prompt, T, top_p, u0)
    if to != tg:
        assert mg <= thr, ("first token", to, tg, mg)
        return 0, 1, 0, 0
    emitted, s, compared, kept, replaced = 1, 0, 0, 0, 0
    while emitted < n_new:
        k_cap = min(max_k, n_new - emitted - 1)
        if k_cap > 0:
            do, co, m1 = o.draft_step_sample(mask, k_cap, eps, T, top_p, U[s, :15])
            dg, cg = g.draft_step_sample(mask, k_cap, eps, T, top_p, U[s, :15])
        else:
            do, dg, m1 = np.zeros(0, np.int32), np.zeros(0, np.int32), 1.0
        if not np.array_equal(do, dg):
            assert m1 <= thr, ("draft", s, do, dg, m1)
            return compared, s + 1, kept, replaced
        if k_cap > 0:
            assert np.allclose(cg, co, rtol=5 * ptol, atol=1e-6)
        block = np.concatenate([[o.pending], do]).astype(np.int32)
        eo, po, m2 = o.verify_sample(block, T, top_p, U[s, 15:30], float(U[s, 30]), want_probs=True)
        eg, pg = g.verify_sample(block, T, top_p, U[s, 15:30], float(U[s, 30]), want_probs=True)
        if not np.array_equal(eo, eg):
            assert m2 <= thr, ("verify", s, eo, eg, m2)
            return compared, s + 1, kept, replaced
        if m2 > thr:      # same nucleus on both sides: the distributions themselves must agree
            rows = len(eo)    # (the oracle stops computing distributions at the first replaced token)
            err = float(np.abs(pg[:rows] - po[:rows]).max())
            assert err <= ptol, (s, err)
            assert np.all(np.abs(pg.sum(axis=1) - 1) < 1e-5)
        assert g.cache_len == o.cache_len and g.pending == o.pending
        compared += int(min(m1, m2) > thr)
        kept += len(eo) - 1
        replaced += int(len(eo) - 1 < len(do))
        emitted += len(eo)
        s += 1
    so, sg = o.stats(), g.stats()
    assert (sg["draft_passes"], sg["verify_passes"], sg["accepted"], sg["emitted_total"]) == \
           (so["draft_passes"], so["verify_passes"], so["accepted"], so["emitted"])
    return compared, s, kept, replaced


@pytest.mark.parametrize("case", list(_CASES))
def test_sampled_decoding_follows_the_oracle(oracle_lib, case):
    shape, max_seq, n_prompt = _CASES[case]
    # (a large vocabulary needs a peaked distribution, or every draw falls within the margin of a boundary)
    weights = hp.shaped_weights(shape, seed=21, head_scale=12.0 if shape.vocab < 1000 else 150.0)
    o, g = _pair(oracle_lib, shape, weights, max_seq)
    prompt = si.uniform_ids(11, n_prompt, shape.vocab)
    rng = np.random.default_rng(9)
    L2 = 2 * shape.n_layers
    masks = [np.zeros(L2, np.uint8), np.ones(L2, np.uint8)] + [(rng.random(L2) < 0.5).astype(np.uint8) for _ in range(2)]
    n_new = 30 if shape.vocab < 1000 else 10
    tot = np.zeros(4, int)
    for i, mask in enumerate(masks):
        for max_k, eps, T, top_p in ((4, 0.0, 0.6, 0.95), (8, 0.2, 1.0, 1.0), (15, 0.0, 0.3, 0.5), (3, 0.0, 1.5, 0.9)):
            U = rng.random((n_new + 2, 31), dtype=np.float32)
            u0 = float(rng.random(dtype=np.float32))
            tot += _lockstep(o, g, shape, prompt, n_new, mask, max_k, eps, T, top_p, u0, U.astype(np.float64))
    compared, steps, kept, replaced = tot
    assert compared >= (0.3 if shape.vocab < 1000 else 0.15) * steps and kept > 0 and replaced > 0, tot
    g.close()


def test_sampled_steps_follow_the_target_distribution_on_gpu(oracle_lib):
    """Many independent steps from one state with fresh uniforms and a layer-skipping draft model: the
    first emitted token follows the target's warped distribution (from the oracle's no-cache forward), not
    the draft's."""
    shape = hp.SMALL_GQA_BF16
    # (strong sublayers: a layer-skipping draft model then differs visibly from the target)
    weights = hp.shaped_weights(shape, seed=21, head_scale=12.0, branch_scale=1.0)
    o, g = _pair(oracle_lib, shape, weights, 96)
    prompt = si.uniform_ids(11, 12, shape.vocab)
    T, top_p = 0.6, 0.95
    mask = np.zeros(2 * shape.n_layers, np.uint8)
    mask[[1, 3, 5]] = 1
    tok0 = g.prefill_sample(prompt, T, top_p, 0.5)
    assert tok0 == o.prefill_sample(prompt, T, top_p, 0.5)[0]
    n0 = g.cache_len
    p1, _ = oracle_lib.warp(o.forward_nocache(list(prompt) + [tok0]), T, top_p)
    q1, _ = oracle_lib.warp(o.forward_row(tok0, n0, mask), T, top_p)
    assert np.abs(p1 - q1).max() > 0.05          # the draft model really differs: the test can tell them apart
    rng = np.random.default_rng(12)
    N = 4000
    first = np.zeros(shape.vocab)
    kept = 0
    for i in range(N):
        g.rollback(n0, tok0)
        u = rng.random(31, dtype=np.float32)
        d, _ = g.draft_step_sample(mask, 2, 0.0, T, top_p, u[:15])
        em, _ = g.verify_sample([tok0] + [int(x) for x in d], T, top_p, u[15:30], float(u[30]))
        first[em[0]] += 1
        kept += len(em) - 1
    sig = np.sqrt(p1 * (1 - p1) / N)
    assert 0 < kept < 2 * N
    assert np.all(np.abs(first / N - p1) <= 5 * sig + 5e-3), np.abs(first / N - p1).max()
    assert np.abs(first / N - q1).max() > 0.03
    g.close()


def test_full_size_sampling_with_the_target_as_draft_keeps_every_token():
    """7B shape, no sublayer skipped: the draft pass computes the target's logits bit for bit (a row's
    logits do not depend on the rows of its pass), so q == p, every draft token is kept, and the output
    is exactly plain sampling fed the same uniforms in order."""
    import paper_2410_06916_amd as P
    w = si.WORKLOADS["7b"]
    shape = w.shape
    n_prompt, n_new, T, top_p = 64, 33, 0.6, 0.95
    g = P.SwiftModel(shape, n_prompt + n_new + 24)
    for nm, t in si.iter_weights(shape, w.weight_seed, "cuda:0"):
        g.load_tensor(nm, t)
    prompt = si.uniform_ids(w.prompt_seed, n_prompt, shape.vocab)
    rng = np.random.default_rng(2)
    U = rng.random((n_new, 31), dtype=np.float32)
    none = np.zeros(2 * shape.n_layers, np.uint8)
    toks, tr = P.generate_swift_sample(g, prompt, n_new, none, 7, 0.0, T, top_p, 0.25, U)
    assert all(t["m"] == len(t["draft"]) for t in tr)
    plain = [g.prefill_sample(prompt, T, top_p, 0.25)]
    for s, t in enumerate(tr):
        for u in list(U[s, :len(t["draft"])]) + [U[s, 30]]:
            em, _ = g.verify_sample([g.pending], T, top_p, [], float(u))
            plain.append(int(em[0]))
    assert plain[:n_new] == [int(x) for x in toks]
    assert len(set(plain)) > 8          # random-init logits at temperature 0.6: the draws really vary
    # with the workload's skip mask the drafts differ from the target: some are replaced, output stays valid
    mask = si.workload_mask(w)
    toks2, tr2 = P.generate_swift_sample(g, prompt, n_new, mask, 7, 0.0, T, top_p, 0.25, U)
    assert toks2.min() >= 0 and toks2.max() < shape.vocab and toks2[0] == toks[0]
    assert 1 + sum(t["m"] + 1 for t in tr2) >= n_new
    g.close()


def test_sampling_errors_on_device(oracle_lib):
    import paper_2410_06916_amd as P
    shape = hp.SMALL_GQA
    weights = hp.shaped_weights(shape, seed=1)
    g = P.SwiftModel(shape, 48)
    g.load_weights(weights)
    prompt = si.uniform_ids(3, 8, shape.vocab)
    mask = np.zeros(2 * shape.n_layers, np.uint8)
    with pytest.raises(P.SwiftError):
        g.prefill_sample(prompt, 0.0, 0.9, 0.5)            # temperature must be positive
    with pytest.raises(P.SwiftError):
        g.prefill_sample(prompt, 0.6, 0.9, 1.0)            # uniform outside [0, 1)
    g.prefill_sample(prompt, 0.6, 0.9, 0.5)
    with pytest.raises(P.SwiftError):
        g.verify_sample([g.pending, 5], 0.6, 0.9, [0.5], 0.5)          # no sampled draft to verify
    d, _ = g.draft_step_sample(mask, 3, 0.0, 0.6, 0.9, [0.1, 0.7, 0.3])
    with pytest.raises(P.SwiftError):
        g.verify_sample([g.pending] + [int(x) for x in d[:2]] + [(int(d[2]) + 1) % shape.vocab], 0.6, 0.9, [0.5] * 3, 0.5)
    with pytest.raises(P.SwiftError):
        g.verify_sample([g.pending] + [int(x) for x in d], 0.6, 0.9, [0.5, -0.1, 0.5], 0.5)
    n0 = g.cache_len
    em, _ = g.verify_sample([g.pending] + [int(x) for x in d[:2]], 0.6, 0.9, [0.5, 0.5], 0.5)   # a prefix is fine
    assert g.cache_len == n0 + len(em) and g.pending == em[-1]
    with pytest.raises(P.SwiftError):
        g.verify_sample([g.pending, int(d[0])], 0.6, 0.9, [0.5], 0.5)     # the distributions are spent
    g.close()


def test_sampled_decoding_on_random_shapes(oracle_lib):
    """The same lockstep comparison on seeded random shapes, temperatures, nucleus sizes, masks and draft
    lengths (head sizes 16..128, vocabularies up to 4000, both storage types)."""
    compared = run = n_done = 0
    for seed in range(30):
        rng = np.random.default_rng(seed + 9000)
        d = int(rng.choice([16, 32, 64, 128]))
        group = int(rng.choice([1, 2, 4]))
        n_kv = int(rng.choice([1, 2]))
        while n_kv * group * d > 512:
            if group > 1:
                group //= 2
            elif n_kv > 1:
                n_kv //= 2
            else:
                d //= 2
        n_q = n_kv * group
        if (n_q * d) % 32:
            continue
        ffn = int(rng.integers(8, 40)) * 8
        vocab = int(rng.integers(50, 2000)) * 2
        dtype = "bf16" if rng.random() < 0.6 else "fp32"
        n_layers = int(rng.integers(1, 4))
        max_seq = int(rng.choice([128, 1700]))
        shape = si.ModelShape(f"random-{seed}", n_layers, n_q * d, n_q, n_kv, d, ffn, vocab, dtype, 1e-5)
        weights = hp.shaped_weights(shape, seed=seed, head_scale=float(rng.choice([20.0, 60.0, 150.0])))
        o, g = _pair(oracle_lib, shape, weights, max_seq)
        prompt = si.uniform_ids(3000 + seed, int(rng.integers(1, 50)), vocab)
        mask = (rng.random(2 * n_layers) < 0.4).astype(np.uint8)
        T = float(rng.choice([0.6, 1.0, 1.5]))
        top_p = float(rng.choice([0.5, 0.9, 0.95, 1.0]))
        max_k = int(rng.integers(1, 15))
        eps = float(rng.choice([0.0, 0.3]))
        U = rng.random((64, 31))
        u0 = float(rng.random())
        c, r, _, _ = _lockstep(o, g, shape, prompt, int(rng.integers(5, 30)), mask, max_k, eps, T, top_p, u0, U)
        compared += c
        run += r
        n_done += 1
        g.close()
        o.close()
    assert n_done >= 20 and compared >= run // 2, (n_done, compared, run)
