"""Pins of the oracle's speculative sampling (Section 5.1, Appendix B.2: speculative sampling as the
acceptance rule, temperature 0.6 and top-p 0.95): the warped distribution against a library softmax
and a brute-force nucleus, inverse-CDF draws against exact interval counts, and the property the
acceptance rule exists for: what a draft-then-verify step emits is distributed exactly as the target
model's own samples, whatever the draft distribution.  CPU only."""
import itertools

import numpy as np
import pytest
from scipy.special import softmax

import synthetic_inputs as si
from tests import helpers as hp


def test_warp_without_nucleus_is_the_tempered_softmax(oracle_lib):
    rng = np.random.default_rng(0)
    for T in (1.0, 0.6, 2.5):
        lg = rng.normal(0, 3, 50)
        p, _ = oracle_lib.warp(lg, T, 1.0)
        assert np.allclose(p, softmax(lg / T), rtol=1e-13, atol=0)
    # temperature -> 0 puts all mass on the arg-max
    p, _ = oracle_lib.warp(np.array([0.3, 1.1, 1.0, -2.0]), 1e-3, 1.0)
    assert np.allclose(p, [0, 1, 0, 0], atol=1e-40)


def test_nucleus_by_hand_and_ties(oracle_lib):
    lg = np.log([0.5, 0.3, 0.15, 0.05])
    assert np.allclose(oracle_lib.warp(lg, 1.0, 0.79)[0], [0.625, 0.375, 0, 0])
    assert np.allclose(oracle_lib.warp(lg, 1.0, 0.81)[0], np.array([0.5, 0.3, 0.15, 0]) / 0.95)
    assert np.allclose(oracle_lib.warp(lg, 1.0, 0.3)[0], [1, 0, 0, 0])           # the top token alone suffices
    assert np.allclose(oracle_lib.warp(lg[::-1].copy(), 1.0, 0.79)[0], [0, 0, 0.375, 0.625])   # order-free
    # the cut falls on a probability that several tokens share: all of them stay
    assert np.allclose(oracle_lib.warp(np.log([0.4, 0.2, 0.2, 0.2]), 1.0, 0.5)[0], [0.4, 0.2, 0.2, 0.2])
    # the margin shrinks as top_p approaches a cumulative sum
    assert oracle_lib.warp(lg, 1.0, 0.81)[1] == pytest.approx(0.01, rel=1e-9)
    assert oracle_lib.warp(lg, 1.0, 0.7999)[1] == pytest.approx(1e-4, rel=1e-6)


def test_nucleus_is_the_smallest_most_probable_set(oracle_lib):
    """Brute force over all subsets of a 12-token vocabulary: the nucleus has the fewest tokens among
    the sets whose mass reaches top_p, and the largest mass among those."""
    rng = np.random.default_rng(1)
    for trial in range(6):
        lg = rng.normal(0, 2, 12)
        T, top_p = (1.0, 0.6, 1.7)[trial % 3], (0.5, 0.9, 0.95, 0.2)[trial % 4]
        full = softmax(lg / T)
        best = None
        for mask in range(1, 1 << 12):
            idx = [i for i in range(12) if mask >> i & 1]
            mass = full[idx].sum()
            if mass >= top_p and (best is None or (len(idx), -mass) < (len(best[0]), -best[1])):
                best = (idx, mass)
        p, _ = oracle_lib.warp(lg, T, top_p)
        assert sorted(np.flatnonzero(p)) == best[0]
        assert np.allclose(p[best[0]], full[best[0]] / best[1], rtol=1e-12)
        assert abs(p.sum() - 1) < 1e-12


def test_inverse_cdf_draws_hit_every_interval_exactly(oracle_lib):
    w = np.array([0.1, 0.0, 0.25, 0.05, 0.0, 0.6]) * 3.0      # unnormalised, with gaps
    N = 20000
    counts = np.zeros(6, int)
    for i in range(N):
        tok, _ = oracle_lib.sample(w, (i + 0.5) / N)
        counts[tok] += 1
    assert np.array_equal(counts, np.round(w / w.sum() * N).astype(int))
    assert oracle_lib.sample(w, 0.0)[0] == 0 and oracle_lib.sample(w, np.nextafter(1.0, 0))[0] == 5
    assert oracle_lib.sample(w, 0.1)[0] == 2          # u on a boundary belongs to the next token


@pytest.mark.parametrize("case", ["overlap", "disjoint-support", "equal", "draft-concentrated"])
def test_one_speculative_step_samples_the_target_distribution(oracle_lib, case):
    """The acceptance rule keeps x ~ q with probability min(1, p(x)/q(x)) and otherwise draws from
    max(0, p - q) renormalised: the emitted token is then distributed as p."""
    rng = np.random.default_rng(3)
    n = 9
    p = rng.dirichlet(np.ones(n))
    if case == "overlap":
        q = rng.dirichlet(np.ones(n))
        p[2] = 0.0
        q[5] = 0.0
    elif case == "disjoint-support":
        q = p.copy()
        p[:4] = 0.0
        q[4:] = 0.0
    elif case == "equal":
        q = p.copy()
    else:
        q = np.full(n, 1e-3)
        q[np.argmin(p)] = 1.0
    p, q = p / p.sum(), q / q.sum()
    N = 1_500_000
    u = rng.random((N, 3))
    out = oracle_lib.spec_first_token_batch(p, q, u)
    freq = np.bincount(out, minlength=n) / N
    sigma = np.sqrt(p * (1 - p) / N)
    assert np.all(np.abs(freq - p) <= 5 * sigma + 1e-12), (freq, p)
    if case == "equal":       # p == q: every draw is kept
        draws = np.array([oracle_lib.sample(q, ui)[0] for ui in u[:2000, 0]])
        assert np.array_equal(out[:2000], draws)
    if case == "disjoint-support":    # nothing can be kept: always the replacement draw from p
        repl = np.array([oracle_lib.sample(p, ui)[0] for ui in u[:2000, 2]])
        assert np.array_equal(out[:2000], repl)


def test_acceptance_and_replacement_by_hand(oracle_lib):
    assert oracle_lib.spec_keep(0.2, 0.4, 0.49) and not oracle_lib.spec_keep(0.2, 0.4, 0.5)
    assert oracle_lib.spec_keep(0.5, 0.4, 0.999999) and not oracle_lib.spec_keep(0.0, 0.4, 0.0)
    p, q = np.array([0.5, 0.1, 0.4]), np.array([0.2, 0.6, 0.2])    # max(0, p - q) = [0.3, 0, 0.2]
    assert oracle_lib.spec_resample(p, q, 0.59) == 0 and oracle_lib.spec_resample(p, q, 0.61) == 2


@pytest.fixture(scope="module")
def small(oracle_lib):
    s = hp.SMALL_GQA
    w = hp.shaped_weights(s, seed=21, head_scale=12.0)
    o = oracle_lib.Oracle(s, 96)
    o.set_weights(w)
    prompt = si.uniform_ids(11, 12, s.vocab)
    return s, o, prompt


def test_sampled_decoding_states_and_degenerate_settings(oracle_lib, small):
    s, o, prompt = small
    T, top_p = 0.6, 0.95
    rng = np.random.default_rng(4)
    U = rng.random((64, oracle_lib.SAMPLE_U_PER_STEP), dtype=np.float32).astype(np.float64)
    none = np.zeros(2 * s.n_layers, np.uint8)
    # the draft model is the target model: q == p, every draft is kept, and the tokens are exactly
    # those of plain sampling that consumes the same draws (draft draw j = plain step j's final draw)
    toks, tr = oracle_lib.generate_swift_sample(o, prompt, 25, none, 4, 0.0, T, top_p, 0.37, U)
    assert all(t["m"] == len(t["draft"]) for t in tr)
    st = o.stats()
    assert st["accepted"] == st["draft_passes"] and st["emitted"] == 25
    # plain sampling: k = 0 steps
    tok0, _ = o.prefill_sample(prompt, T, top_p, 0.37)
    assert tok0 == toks[0]
    seq = [tok0]
    i = 0
    for t in tr:
        for u in list(U[i, :len(t["draft"])]) + [U[i, 30]]:
            em, pr, _ = o.verify_sample([o.pending], T, top_p, [], float(u), want_probs=True)
            assert len(em) == 1 and abs(pr.sum() - 1) < 1e-12
            seq.append(int(em[0]))
        i += 1
    assert seq[:25] == [int(x) for x in toks]
    # first token: the warped distribution of the brute-force (no cache) logits, drawn with u0
    p0, _ = oracle_lib.warp(o.forward_nocache(prompt), T, top_p)
    assert tok0 == oracle_lib.sample(p0, 0.37)[0]
    # state after a step: cache length n + m + 1, pending = last emitted; errors
    o.prefill_sample(prompt, T, top_p, 0.5)
    mask = np.ones(2 * s.n_layers, np.uint8)
    d, conf, _ = o.draft_step_sample(mask, 5, 0.0, T, top_p, U[0, :15])
    n0 = o.cache_len
    with pytest.raises(oracle_lib.OracleError):
        o.verify_sample([o.pending] + [int(x) for x in d[:-1]] + [int(d[-1]) ^ 1], T, top_p, U[0, 15:30], 0.1)
    em, _, _ = o.verify_sample([o.pending] + [int(x) for x in d], T, top_p, U[0, 15:30], 0.1)
    assert o.cache_len == n0 + len(em) and o.pending == em[-1]
    assert np.array_equal(em[:-1], d[:len(em) - 1])
    with pytest.raises(oracle_lib.OracleError):       # the draft distributions are gone after the step
        o.verify_sample([o.pending, 3], T, top_p, U[0, 15:30], 0.1)


def test_sampled_speculation_matches_the_target_model_in_distribution(oracle_lib, small):
    """Many independent decoding steps from the same state, each with fresh uniforms and a
    layer-skipping draft model: the first emitted token follows the target's warped distribution
    computed by brute force (no cache), and, among the runs that start with the most likely token,
    so does the second."""
    s, o, prompt = small
    T, top_p = 0.6, 0.95
    rng = np.random.default_rng(6)
    mask = np.zeros(2 * s.n_layers, np.uint8)
    mask[[1, 2, 5]] = 1
    tok0, _ = o.prefill_sample(prompt, T, top_p, 0.5)
    n0 = o.cache_len
    p1, _ = oracle_lib.warp(o.forward_nocache(list(prompt) + [tok0]), T, top_p)
    t1 = int(np.argmax(p1))
    p2, _ = oracle_lib.warp(o.forward_nocache(list(prompt) + [tok0, t1]), T, top_p)
    N = 6000
    first = np.zeros(s.vocab)
    second = np.zeros(s.vocab)
    kept = rejected = 0
    for i in range(N):
        o.rollback(n0, tok0)
        u = rng.random(oracle_lib.SAMPLE_U_PER_STEP)
        d, _, _ = o.draft_step_sample(mask, 2, 0.0, T, top_p, u[:15])
        em, _, _ = o.verify_sample([tok0] + [int(x) for x in d], T, top_p, u[15:30], float(u[30]))
        kept += len(em) - 1
        rejected += len(em) - 1 < len(d)
        first[em[0]] += 1
        if em[0] == t1:
            if len(em) == 1:       # the step ended on the first token: one more plain step
                em = np.concatenate([em, o.verify_sample([o.pending], T, top_p, [], float(rng.random()))[0]])
            second[em[1]] += 1
    assert kept > N // 4 and rejected > N // 20          # both branches of the rule are exercised
    assert np.count_nonzero(p1) > 3 and np.count_nonzero(p2) > 3
    sig1 = np.sqrt(p1 * (1 - p1) / N)
    assert np.all(np.abs(first / N - p1) <= 5 * sig1 + 1e-9), np.abs(first / N - p1).max()
    n2 = second.sum()
    sig2 = np.sqrt(p2 * (1 - p2) / n2)
    assert n2 > N // 10 and np.all(np.abs(second / n2 - p2) <= 5 * sig2 + 1e-9)
