"""Pins of the oracle's decoding loop: the lossless invariant (speculative greedy
output == plain greedy output of the target model; Sections 1 and 3.1 state that
verification leaves the output unchanged), brute-force recomputation without a
cache, the degenerate settings of the method, and the counter identities behind
M and alpha (Appendix B.3).  CPU only."""
import numpy as np
import pytest

import synthetic_inputs as si
from tests import helpers as hp


@pytest.fixture(scope="module")
def small(oracle_lib):
    s = hp.SMALL_GQA
    w = hp.shaped_weights(s, seed=21)
    o = oracle_lib.Oracle(s, 96)
    o.set_weights(w)
    prompt = si.uniform_ids(11, 12, s.vocab)
    ar = oracle_lib.generate_ar(o, prompt, 40)
    return s, o, prompt, ar


def _masks(n_layers):
    L2 = 2 * n_layers
    rng = np.random.default_rng(5)
    out = {"none": np.zeros(L2, np.uint8), "all": np.ones(L2, np.uint8)}
    for i in range(L2):
        m = np.zeros(L2, np.uint8)
        m[i] = 1
        out[f"only{i}"] = m
    for j in range(4):
        out[f"rand{j}"] = (rng.random(L2) < 0.5).astype(np.uint8)
    return out


def test_cached_forward_equals_bruteforce_bitwise(oracle_lib, small):
    s, o, prompt, ar = small
    seq = np.concatenate([prompt, ar])[:30]
    o.reset()
    for t, tok in enumerate(seq):
        cached = o.forward_row(int(tok), t)
        if t in (0, 1, 2, 7, 13, 29):
            assert np.array_equal(cached, o.forward_nocache(seq[:t + 1])), t


def test_ar_tokens_equal_bruteforce_greedy(oracle_lib, small):
    s, o, prompt, ar = small
    seq = list(prompt)
    for i in range(10):
        tok, _ = oracle_lib.argmax_conf(o.forward_nocache(seq))
        assert tok == ar[i]
        seq.append(tok)


@pytest.mark.parametrize("max_k,eps", [(1, 0.0), (3, 0.0), (4, 0.5), (7, 0.8), (5, 2.0)])
def test_speculative_equals_autoregressive(oracle_lib, small, max_k, eps):
    s, o, prompt, ar = small
    seen_partial = False
    for name, mask in _masks(s.n_layers).items():
        out, trace = oracle_lib.generate_swift(o, prompt, len(ar), mask, max_k, eps)
        assert np.array_equal(out, ar), (name, max_k, eps)
        for st in trace:
            k = len(st["draft"])
            seen_partial |= 0 < st["m"] < k
            # what was emitted: the accepted drafts, then the target's own token
            assert list(st["emitted"][:-1]) == list(st["draft"][:st["m"]])
            assert st["emitted"][-1] == st["target"][st["m"]]
            assert st["m"] == k or st["draft"][st["m"]] != st["target"][st["m"]]
    if max_k >= 3 and eps < 1:
        assert seen_partial      # the inputs do exercise partial acceptance (0 < m < k)


def test_poisoned_slots_beyond_cache_length_are_never_read(oracle_lib, small):
    s, o, prompt, ar = small
    for name, mask in list(_masks(s.n_layers).items())[:6]:
        out, _ = oracle_lib.generate_swift(o, prompt, len(ar), mask, 4, 0.3, poison=True)
        assert np.array_equal(out, ar), name


def test_no_skip_mask_accepts_everything(oracle_lib, small):
    s, o, prompt, ar = small
    n_new, max_k = 33, 4
    out, trace = oracle_lib.generate_swift(o, prompt, n_new, np.zeros(2 * s.n_layers, np.uint8), max_k, 0.0)
    assert np.array_equal(out, ar[:n_new])
    assert all(st["m"] == len(st["draft"]) for st in trace)
    # eps = 0: every step drafts max_k tokens until the cap "tokens still wanted - 1" bites
    assert [len(st["draft"]) for st in trace][:-1] == [max_k] * (len(trace) - 1)
    st = o.stats()
    assert st["accepted"] == st["draft_passes"]                          # alpha = 1
    assert st["emitted"] == n_new
    assert len(trace) == -(-(n_new - 1) // (max_k + 1))                  # M = max_k + 1 per full step


def test_threshold_extremes_and_zero_draft_length(oracle_lib, small):
    s, o, prompt, ar = small
    mask = _masks(s.n_layers)["rand1"]
    _, trace = oracle_lib.generate_swift(o, prompt, 20, mask, 5, 2.0)    # eps > 1: stop after one draft
    assert all(len(st["draft"]) <= 1 for st in trace)
    assert all(len(st["draft"]) == 1 for st in trace[:-1])
    _, trace = oracle_lib.generate_swift(o, prompt, 20, mask, 5, 0.0)    # eps = 0: never stops early
    assert all(len(st["draft"]) == min(5, 20 - 1 - sum(len(t["emitted"]) for t in trace[:i]) - 1)
               for i, st in enumerate(trace))
    out, trace = oracle_lib.generate_swift(o, prompt, 20, mask, 0, 0.5)  # no drafting = vanilla, M = 1
    assert np.array_equal(out, ar[:20]) and len(trace) == 19 and o.stats()["draft_passes"] == 0


def test_early_stop_keeps_the_low_confidence_token(oracle_lib, small):
    s, o, prompt, ar = small
    mask = _masks(s.n_layers)["rand0"]
    _, trace = oracle_lib.generate_swift(o, prompt, 40, mask, 6, 0.6)
    stops = 0
    for st in trace:
        c = st["conf"]
        assert np.all(c[:-1] >= 0.6)          # drafting went on only while confident
        if len(c) < 6 and len(c) > 0 and c[-1] < 0.6:
            stops += 1                        # the sub-threshold token is in the verified block
            assert len(st["block"]) == len(c) + 1
    assert stops > 0
    assert np.all((0 < np.concatenate([st["conf"] for st in trace])) &
                  (np.concatenate([st["conf"] for st in trace]) <= 1))


def test_counter_identities(oracle_lib, small):
    s, o, prompt, ar = small
    out, trace = oracle_lib.generate_swift(o, prompt, 37, _masks(s.n_layers)["rand2"], 4, 0.4)
    st = o.stats()
    assert st["emitted"] == 37 == len(out)
    assert st["verify_passes"] == len(trace)
    assert st["draft_passes"] == sum(len(t["draft"]) for t in trace)
    assert st["accepted"] == sum(t["m"] for t in trace)
    assert 1 + sum(t["m"] + 1 for t in trace) == 37       # prefill's token + (m+1) per target pass
    assert o.cache_len == len(prompt) + 36                 # everything but the pending token is cached
    assert o.pending == out[-1]


def test_verify_block_rows_equal_single_row_forwards(oracle_lib, small):
    """Row i of a verify block is the target's forward of that token at position
    n+i: the same logits, bit for bit, as decoding the block one token at a time."""
    s, o, prompt, ar = small
    o.prefill(prompt)
    block = np.array([o.pending, 5, 9, 150], np.int32)
    tgt, lg = o.verify(block, want_logits=True)
    o2 = oracle_lib.Oracle(s, 96)
    o2._keep = o._keep
    o2.set_weights(o._keep)
    want = o2.forward_nocache(np.concatenate([prompt, block]))
    assert np.array_equal(lg[3], want)
    assert tgt[3] == oracle_lib.argmax_conf(want)[0]


def _decode_to(o, oracle_lib, prompt, n_tokens):
    """Greedy-decodes n_tokens tokens; returns the whole sequence prompt + generated (the last
    generated token is the pending one)."""
    out = oracle_lib.generate_ar(o, prompt, n_tokens)
    return np.concatenate([np.asarray(prompt, np.int32), out])


def test_candidate_evaluation_empty_set_scores_every_token(oracle_lib, small):
    """Section 4.1.2, Eq. 3-4: with nothing skipped the draft model is the target model reading
    the target's own cache, so it reproduces each of the last gamma generated tokens: matchness 1
    exactly.  (A wrong position, a window shifted by one, an attention range one slot short or long,
    or recomputed instead of reused keys would all break the equality with the generated tokens.)"""
    s, o, prompt, ar = small
    seq = _decode_to(o, oracle_lib, prompt, 30)
    none = np.zeros(2 * s.n_layers, np.uint8)
    for gamma in (1, 7, 29):
        pred, n_match = o.eval_mask(none, seq[-(gamma + 1):])
        assert n_match == gamma and np.array_equal(pred, seq[-gamma:])
    # the logits of a row are those the target produced when it generated that token
    n = o.cache_len
    pred, n_match, lg = o.eval_mask(none, seq[-4:], want_logits=True)
    o2 = oracle_lib.Oracle(s, 96)
    o2.set_weights(hp.shaped_weights(s, seed=21))
    o2.prefill(seq[:n - 2])                      # pending = seq[n - 2]
    _, lg2 = o2.verify([o2.pending], True)       # row at position n - 2 predicts seq[n - 1]
    assert np.array_equal(lg[1], lg2[0])
    o2.close()


def test_candidate_evaluation_all_skipped_closed_form(oracle_lib, small):
    """Everything skipped: prediction i is arg-max W_lm . rmsnorm(E[window[i-1]]), whatever the
    context; matchness counts the agreements with the generated tokens."""
    s, o, prompt, ar = small
    seq = _decode_to(o, oracle_lib, prompt, 20)
    w = {k: v.double().numpy() for k, v in hp.shaped_weights(s, seed=21).items()}
    allm = np.ones(2 * s.n_layers, np.uint8)
    window = seq[-11:]
    pred, n_match = o.eval_mask(allm, window)
    want = []
    for t in window[:-1]:
        x = w["embed"][t]
        xh = x / np.sqrt(np.mean(x * x) + s.rms_eps) * w["final_norm"]
        want.append(int(np.argmax((w["lm_head"] @ xh).astype(np.float32))))
    assert np.array_equal(pred, want)
    assert n_match == int(np.sum(np.array(want) == window[1:]))


def test_candidate_evaluation_reads_only_earlier_slots_and_changes_nothing(oracle_lib, small):
    """A row's prediction depends on cache slots up to its own position only (the same rows
    evaluated from a shorter cache give the same logits), and the evaluation leaves cache, length,
    pending token and the continuation untouched."""
    s, o, prompt, ar = small
    masks = _masks(s.n_layers)
    seq = _decode_to(o, oracle_lib, prompt, 24)
    n, pend = o.cache_len, o.pending
    kv_before = [o.read_kv(l, p) for l in range(s.n_layers) for p in (0, n - 5, n - 1)]
    o2 = oracle_lib.Oracle(s, 96)
    o2.set_weights(hp.shaped_weights(s, seed=21))
    assert o2.prefill(seq[:n - 3])[0] == seq[n - 3]
    for name in ("rand0", "rand1", "only0", "only1", "only2", "only5"):
        m = masks[name]
        pred, n_match, lg = o.eval_mask(m, seq[-9:], want_logits=True)      # rows at positions n-8 .. n-1
        assert (o.cache_len, o.pending) == (n, pend)
        # the same rows from a cache that is three tokens shorter: positions n-8 .. n-4
        pred2, _, lg2 = o2.eval_mask(m, seq[n - 8:n - 2], want_logits=True)
        assert np.array_equal(lg2, lg[:5]) and np.array_equal(pred2, pred[:5])
        assert 0 <= n_match <= 8 and n_match == int(np.sum(pred == seq[-8:]))
        # nothing was written: a draft model that recomputed the window's keys and values would leave
        # its own in the slots of the layers behind a skipped sublayer
        kv_after = [o.read_kv(l, p) for l in range(s.n_layers) for p in (0, n - 5, n - 1)]
        for (k0, v0), (k1, v1) in zip(kv_before, kv_after):
            assert np.array_equal(k0, k1) and np.array_equal(v0, v1), name
    tgt, _ = o.verify([o.pending])
    o.accept()
    assert int(tgt[0]) == int(oracle_lib.generate_ar(o, prompt, 26)[24])
    # window longer than the cache, evaluation before prefill
    with pytest.raises(Exception):
        o.eval_mask(masks["none"], np.zeros(o.cache_len + 2, np.int32))
    o2.close()


def test_layer_set_suggestion_candidates(oracle_lib):
    """Section 4.1.2, Eq. 2 (random search under a fixed skip ratio r) and Section 4.1.1 (uniform
    initial pattern): every candidate skips exactly round(r L) sublayers, all of them eligible; the
    stream is a function of (seed, step) only; every eligible sublayer is picked about equally
    often; the initial pattern is evenly spaced."""
    el = np.zeros(64, np.uint8)
    el[4:60] = 1                                     # layers 2..29 of 32
    opt = oracle_lib.Optimizer(64, 0.5, seed=7, eligible=el)
    again = oracle_lib.Optimizer(64, 0.5, seed=7, eligible=el)
    other = oracle_lib.Optimizer(64, 0.5, seed=8, eligible=el)
    counts = np.zeros(64)
    differs = 0
    for step in range(2, 2002):
        c = opt.candidate(step)
        assert c.sum() == 32 and not np.any(c[el == 0])
        assert np.array_equal(c, again.candidate(step))
        differs += int(not np.array_equal(c, other.candidate(step)))
        counts += c
    assert differs > 1990
    freq = counts[4:60] / 2000.0                     # expected 32/56 each, binomial sd 0.011
    assert np.all(np.abs(freq - 32 / 56) < 0.05)
    assert len({opt.candidate(s).tobytes() for s in range(2, 200)}) > 190
    # evenly spaced initial pattern: every other sublayer for r = 1/2 over all, and inside a range
    assert np.array_equal(oracle_lib.Optimizer(8, 0.5).initial_mask(), [0, 1, 0, 1, 0, 1, 0, 1])
    init = opt.initial_mask()
    assert init.sum() == 32 and not np.any(init[el == 0])
    gaps = np.diff(np.nonzero(init)[0])
    assert gaps.min() >= 1 and gaps.max() <= 2
    assert oracle_lib.Optimizer(10, 0.0).initial_mask().sum() == 0
    with pytest.raises(Exception):
        oracle_lib.Optimizer(8, 0.9, eligible=np.array([1, 1, 0, 0, 0, 0, 0, 0], np.uint8))
    for o in (opt, again, other):
        o.close()


def test_optimisation_steps_retain_the_best_and_terminate(oracle_lib, small):
    """Bookkeeping and termination of the optimisation phase (Section 4.1.2, Appendix B.2): step 1
    scores the uniform pattern, later steps random candidates; each score is the matchness of that
    candidate on the window; the retained set is the first best so far; the phase ends at the step
    limit, after max_stale steps without improvement, or when the best matchness exceeds the bound."""
    s, o, prompt, ar = small
    seq = _decode_to(o, oracle_lib, prompt, 40)
    window = seq[-17:]
    L2 = 2 * s.n_layers

    def run(**kw):
        opt = oracle_lib.Optimizer(L2, **kw)
        hist = []
        while True:
            r = opt.step(o, window)
            hist.append(r)
            if r["finished"]:
                break
        with pytest.raises(Exception):
            opt.step(o, window)                       # finished: no more steps
        first, cand2 = opt.initial_mask(), opt.candidate(2)
        opt.close()
        return hist, first, cand2

    hist, first, cand2 = run(skip_ratio=0.5, max_steps=12, max_stale=100, stop_matchness=2.0, seed=3)
    assert len(hist) == 12                            # step limit
    assert np.array_equal(hist[0]["candidate"], first) and np.array_equal(hist[1]["candidate"], cand2)
    best, best_mask = -1.0, None
    for r in hist:
        pred, n_match = o.eval_mask(r["candidate"], window)
        assert r["score"] == n_match / 16
        if r["score"] > best:
            best, best_mask = r["score"], r["candidate"]
        assert r["best_score"] == best and np.array_equal(r["best"], best_mask)
    # nothing improves on a perfect first score: stops after max_stale further steps
    hist, _, _ = run(skip_ratio=0.0, max_steps=50, max_stale=4, stop_matchness=2.0, seed=3)
    assert hist[0]["score"] == 1.0 and len(hist) == 5 and all(r["best_score"] == 1.0 for r in hist)
    # matchness above the bound ends the phase at once (the paper's 0.95)
    hist, _, _ = run(skip_ratio=0.0, max_steps=50, max_stale=4, stop_matchness=0.95, seed=3)
    assert len(hist) == 1 and hist[0]["finished"]
    # "exceeds": a score equal to the bound does not stop it
    hist, _, _ = run(skip_ratio=0.0, max_steps=3, max_stale=100, stop_matchness=1.0, seed=3)
    assert len(hist) == 3


def test_topk_widths_and_selection(oracle_lib):
    """Section 4.2, strategy 2: k = 10, 5, 3, 1 for a confidence in (0, 0.5], (0.5, 0.8], (0.8, 0.95],
    (0.95, 1]; the k candidates are the k largest logits, largest first, equal values in index order."""
    L = oracle_lib.lib()
    for p, k in ((1e-9, 10), (0.3, 10), (0.5, 10), (0.50001, 5), (0.8, 5), (0.80001, 3), (0.95, 3), (0.950001, 1),
                 (1.0, 1)):
        assert L.ora_topk_width(p) == k, p
    rng = np.random.default_rng(0)
    import ctypes as C
    for n in (12, 200, 1000):
        lg = rng.normal(size=n)
        lg[rng.integers(0, n, 6)] = lg[3]                   # ties
        out = np.zeros(10, np.int32)
        L.ora_topk(lg.ctypes.data_as(C.POINTER(C.c_double)), n, 10, out.ctypes.data_as(C.POINTER(C.c_int32)))
        want = np.argsort(-lg.astype(np.float32), kind="stable")[:10]
        assert np.array_equal(out, want)


@pytest.mark.parametrize("max_k,eps", [(1, 0.0), (4, 0.0), (8, 0.6), (15, 0.3)])
def test_dynamic_verification_is_lossless(oracle_lib, small, max_k, eps):
    """Sections 1 and 3.1: whatever is drafted, and however widely it is verified, the output is the
    target model's greedy output.  Also: the cache that tree acceptance leaves behind (accepted rows
    moved to consecutive slots) is the cache plain decoding builds; a block never exceeds 32 rows;
    the counters add up."""
    s, o, prompt, ar = small
    masks = _masks(s.n_layers)
    ref = oracle_lib.Oracle(s, 96)
    ref.set_weights(hp.shaped_weights(s, seed=21))
    leaf_hits = 0
    for name in ("none", "all", "only1", "only4", "rand0", "rand2"):
        out, trace = oracle_lib.generate_swift_tree(o, prompt, 40, masks[name], max_k, eps)
        assert np.array_equal(out, ar), name
        assert 1 + sum(t["m"] + 1 for t in trace) == 40
        for t in trace:
            rows = 1 + sum(len(l) for l in t["levels"])
            assert rows <= oracle_lib.Oracle.TREE_ROWS == 32 and len(t["levels"]) <= max_k
            for lev, p in zip(t["levels"], t["conf"]):
                assert 1 <= len(lev) <= oracle_lib.lib().ora_topk_width(p) and len(set(lev.tolist())) == len(lev)
            # an accepted candidate beside the spine ends the path
            path = t["emitted"][:-1]
            for j, tok in enumerate(path):
                assert tok in t["levels"][j]
                if tok != t["levels"][j][0]:
                    assert j == len(path) - 1
                    leaf_hits += 1
        # the cache equals the one plain decoding leaves (same rows, same arithmetic, moved)
        n = o.cache_len
        ref.prefill(np.concatenate([prompt, out])[:n])
        for l in range(s.n_layers):
            for pos in (n - 1, n - 2, n - 5, n - 9):
                ko, vo = o.read_kv(l, pos)
                kr, vr = ref.read_kv(l, pos)
                assert np.array_equal(ko, kr) and np.array_equal(vo, vr), (name, l, pos)
    if max_k >= 4:
        assert leaf_hits > 0          # the widening really rescued some positions
    ref.close()


def test_width_one_tree_is_the_plain_chain(oracle_lib, small):
    """With one candidate per position the token tree is the draft chain: same drafts, same target
    tokens, same accepted counts, same logits as ora_verify, step by step."""
    s, o, prompt, ar = small
    masks = _masks(s.n_layers)
    for name in ("rand1", "only3"):
        out_c, tr_c = oracle_lib.generate_swift(o, prompt, 30, masks[name], 5, 0.4)
        out_t, tr_t = oracle_lib.generate_swift_tree(o, prompt, 30, masks[name], 5, 0.4, max_width=1)
        assert np.array_equal(out_c, out_t) and len(tr_c) == len(tr_t)
        for c, t in zip(tr_c, tr_t):
            assert np.array_equal(c["draft"], [l[0] for l in t["levels"]])
            assert np.array_equal(c["target"], t["target"]) and c["m"] == t["m"]
    # a wider tree never accepts fewer tokens per step at the same state than the chain would
    o.prefill(prompt)
    levels, conf = o.draft_step_topk(masks["rand1"], 5, 0.0)
    tgt, lg_t = o.verify_tree(o.pending, levels, want_logits=True)
    spine_rows = np.cumsum([1] + [len(l) for l in levels[:-1]])
    chain = np.array([o.pending] + [l[0] for l in levels], np.int32)
    o.accept_tree()
    o.prefill(prompt)
    tgt_c, lg_c = o.verify(chain, True)
    assert np.array_equal(lg_c[0], lg_t[0])
    for j, r in enumerate(spine_rows):
        assert np.array_equal(lg_c[j + 1], lg_t[r])       # spine rows see exactly the chain's context
    o.accept()


def test_tree_acceptance_by_hand(oracle_lib, small):
    """Hand-built trees: a candidate beside the spine is accepted and ends the path even when the
    next level happens to hold the token that follows it (that level continues the spine, not the
    accepted candidate); a spine hit goes on to the next level; no hit emits only the target's token."""
    s, o, prompt, ar = small
    g0, g1, g2 = int(ar[1]), int(ar[2]), int(ar[3])
    wrong = (g0 + 1) % s.vocab
    other = (g1 + 7) % s.vocab
    n0 = len(prompt)
    # accepted beside the spine at level 1; level 2 (children of `wrong`) contains g1
    o.prefill(prompt)
    o.verify_tree(o.pending, [np.array([wrong, g0], np.int32), np.array([g1, other], np.int32)])
    assert np.array_equal(o.accept_tree(), [g0, g1]) and (o.cache_len, o.pending) == (n0 + 2, g1)
    # spine hits at both levels, then the target's own token
    o.prefill(prompt)
    o.verify_tree(o.pending, [np.array([g0, wrong], np.int32), np.array([g1, other], np.int32)])
    assert np.array_equal(o.accept_tree(), [g0, g1, g2]) and (o.cache_len, o.pending) == (n0 + 3, g2)
    # spine hit at level 1, a candidate beside the spine at level 2
    o.prefill(prompt)
    o.verify_tree(o.pending, [np.array([g0, wrong], np.int32), np.array([other, g1], np.int32)])
    assert np.array_equal(o.accept_tree(), [g0, g1, g2]) and o.cache_len == n0 + 3
    # nothing matches
    o.prefill(prompt)
    o.verify_tree(o.pending, [np.array([wrong], np.int32), np.array([g1], np.int32)])
    assert np.array_equal(o.accept_tree(), [g0]) and (o.cache_len, o.pending) == (n0 + 1, g0)
    # decoding continues correctly from the compacted cache
    tgt, _ = o.verify([o.pending])
    assert int(tgt[0]) == g1
    o.accept()
    with pytest.raises(Exception):
        o.accept_tree()                                # no tree outstanding
    with pytest.raises(Exception):
        o.verify_tree(o.pending, [np.arange(10, dtype=np.int32)] * 3 + [np.arange(2, dtype=np.int32)])   # 33 rows


def test_tree_blocks_shrink_to_the_cache_slots_left(oracle_lib, small):
    """Every row of a tree block takes a cache slot of its own, so a block holds at most
    min(32, capacity - cache length) rows: with a cache that has room for only a few slots beyond the
    generated tokens the candidate sets are narrowed, never refused, and the output stays the target
    model's greedy output (Sections 1 and 3.1); with no slot left drafting is refused."""
    s, _, prompt, ar = small
    n_new = 40
    tight = oracle_lib.Oracle(s, len(prompt) + n_new + 2)
    tight.set_weights(hp.shaped_weights(s, seed=21))
    masks = _masks(s.n_layers)
    narrowed = 0
    for name in ("all", "rand0"):
        out, trace = oracle_lib.generate_swift_tree(tight, prompt, n_new, masks[name], 8, 0.0)
        assert np.array_equal(out, ar), name
        for t in trace:
            rows = 1 + sum(len(l) for l in t["levels"])
            assert rows <= min(32, len(prompt) + n_new + 2 - t["n"])
            narrowed += int(rows == len(prompt) + n_new + 2 - t["n"])
    assert narrowed > 0
    # fill the cache to the last slot: no room for the pending token's row
    tight.prefill(prompt)
    while tight.cache_len < len(prompt) + n_new + 2:
        tight.verify([tight.pending]); tight.accept()
    with pytest.raises(oracle_lib.OracleError):
        tight.draft_step_topk(masks["all"], 3, 0.0)
    tight.close()


@pytest.mark.parametrize("tree_width", [0, 10])
def test_whole_method_phases_and_losslessness(oracle_lib, small, tree_width):
    """Section 4 end to end: context accumulation with the uniform pattern, one optimisation step before
    every decoding step once gamma generated tokens are committed, acceleration with the retained set
    after termination; the output equals plain greedy decoding throughout."""
    s, o, prompt, ar = small
    L2 = 2 * s.n_layers
    gamma = 6
    opt = oracle_lib.Optimizer(L2, skip_ratio=0.5, max_steps=4, max_stale=100, stop_matchness=2.0, seed=3)
    toks, tr = oracle_lib.generate_swift_on_the_fly(o, opt, prompt, 40, 5, 0.3, gamma=gamma, tree_width=tree_width)
    assert np.array_equal(toks, ar)
    emitted = 1
    steps = []
    for t in tr:
        if t["opt"] is None:
            # no optimisation step: either the window is not full yet, or the phase is over
            assert emitted - 1 < gamma or len(steps) == 4
            if emitted - 1 < gamma:
                assert np.array_equal(t["mask"], opt.initial_mask())
        else:
            assert emitted - 1 >= gamma and len(steps) < 4
            steps.append(t["opt"])
            assert np.array_equal(t["mask"], t["opt"]["best"])       # the retained set drafts this very step
        emitted += len(t["emitted"])
    assert len(steps) == 4 and steps[-1]["finished"] and not steps[-2]["finished"]
    assert np.array_equal(steps[0]["candidate"], opt.initial_mask())
    best = max(x["score"] for x in steps)
    assert steps[-1]["best_score"] == best
    assert all(np.array_equal(t["mask"], steps[-1]["best"]) for t in tr[-3:])   # acceleration phase
    opt.close()


def test_state_and_capacity_errors(oracle_lib, small):
    s, o, prompt, ar = small
    o.reset()
    with pytest.raises(oracle_lib.OracleError) as e:
        o.verify([1])
    assert e.value.code == -3
    o.prefill(prompt)
    with pytest.raises(oracle_lib.OracleError) as e:
        o.accept()
    assert e.value.code == -3
    with pytest.raises(oracle_lib.OracleError) as e:
        o.draft_step(np.zeros(2 * s.n_layers, np.uint8), 96, 0.5)
    assert e.value.code in (-1, -2)


def test_tiny_workload_runs_and_is_lossless(oracle_lib):
    w = si.WORKLOADS["tiny"]
    o = oracle_lib.Oracle(w.shape, w.n_prompt + w.n_new + w.max_k + 1)
    o.set_weights(si.make_weights(w.shape, w.weight_seed))
    prompt = si.workload_prompt(w)
    ar = oracle_lib.generate_ar(o, prompt, w.n_new)
    for eps in (w.conf_threshold, 0.0):
        out, _ = oracle_lib.generate_swift(o, prompt, w.n_new, si.workload_mask(w), w.max_k, eps)
        assert np.array_equal(out, ar)
