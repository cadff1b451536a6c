"""GPU parity on seeded random model shapes: head sizes 16..128, 1..8 query heads per kv head, ragged FFN
and vocabulary sizes, both storage types, cache capacities on either side of the attention kernels' switch
points, prompt lengths that give every block size.  Each case: prefill, one verify block of 1..12 rows
(logits against the oracle, to the tolerance of the storage type), one candidate evaluation over a window
of up to 99 tokens (predictions equal wherever the oracle's arg-max is not a near tie)."""
import numpy as np
import pytest

import synthetic_inputs as si
from tests import helpers as hp

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def _random_case(seed):
    rng = np.random.default_rng(seed)
    d = int(rng.choice([16, 32, 64, 128]))
    group = int(rng.choice([1, 2, 4, 8]))
    n_kv = int(rng.choice([1, 2, 4]))
    while n_kv * group * d > 1024:
        if group > 1:
            group //= 2
        elif n_kv > 1:
            n_kv //= 2
        else:
            d //= 2
    n_q = n_kv * group
    hidden = n_q * d
    ffn = int(rng.integers(8, 60)) * 8
    vocab = int(rng.integers(50, 350)) * 2
    dtype = "bf16" if rng.random() < 0.7 else "fp32"
    max_seq = int(rng.choice([96, 400, 1700, 2100]))
    n_prompt = int(rng.integers(1, min(330, max_seq - 40)))
    shape = si.ModelShape(f"random-{seed}", 2, hidden, n_q, n_kv, d, ffn, vocab, dtype, 1e-5)
    return rng, shape, max_seq, n_prompt


@pytest.mark.parametrize("first_seed", [0, 30, 60])
def test_random_shapes_against_oracle(oracle_lib, first_seed):
    import paper_2410_06916_amd as P
    n_done = 0
    for seed in range(first_seed, first_seed + 30):
        rng, shape, max_seq, n_prompt = _random_case(seed)
        if shape.hidden % 32:
            continue
        what = (seed, shape, max_seq, n_prompt)
        weights = hp.shaped_weights(shape, seed=seed)
        o = oracle_lib.Oracle(shape, max_seq, threads=8)
        o.set_weights(weights)
        g = P.SwiftModel(shape, max_seq)
        g.load_weights(weights)
        prompt = si.uniform_ids(1000 + seed, n_prompt, shape.vocab)
        _, last_row = o.prefill(prompt)
        g.prefill(prompt)
        if g.pending != o.pending:
            # only a near tie of the oracle's own logits may fall the other way; then follow the oracle
            assert hp.top2_margin(last_row) <= TOL[shape.dtype], (what, hp.top2_margin(last_row))
            g.rollback(g.cache_len, int(o.pending))
        k = int(rng.integers(0, 12))
        block = [int(o.pending)] + [int(x) for x in rng.integers(0, shape.vocab, k)]
        _, lo_ = o.verify(block, True)
        _, lg = g.verify(block, True)
        assert np.all(hp.rel_err_rowmax(lg, lo_) <= TOL[shape.dtype]), what
        gamma = int(min(n_prompt, rng.integers(1, 100)))
        window = np.concatenate([prompt[-gamma:], [o.pending]]).astype(np.int32)
        o.rollback(n_prompt, int(o.pending))
        g.rollback(n_prompt, int(o.pending))
        mask = (rng.random(4) < 0.4).astype(np.uint8)
        po, _, lgo = o.eval_mask(mask, window, want_logits=True)
        pg, _ = g.eval_mask(mask, window)
        srt = np.sort(lgo, axis=1)
        clear = (srt[:, -1] - srt[:, -2]) > (1e-3 if shape.dtype == "bf16" else 1e-5) * np.abs(lgo).max(axis=1)
        assert np.array_equal(np.asarray(pg)[clear], np.asarray(po)[clear]), what
        g.close()
        o.close()
        n_done += 1
    assert n_done >= 20


def _random_loop_case(seed, dtype):
    rng = np.random.default_rng(seed + 7000)
    d = int(rng.choice([16, 32, 64, 128]))
    group = int(rng.choice([1, 2, 4, 8]))
    n_kv = int(rng.choice([1, 2, 4]))
    while n_kv * group * d > 512:
        if group > 1:
            group //= 2
        elif n_kv > 1:
            n_kv //= 2
        else:
            d //= 2
    n_q = n_kv * group
    ffn = int(rng.integers(8, 40)) * 8
    vocab = int(rng.integers(50, 300)) * 2
    n_layers = int(rng.integers(2, 5))
    max_seq = int(rng.choice([128, 1700]))
    n_prompt = int(rng.integers(1, 60))
    n_new = int(rng.integers(4, 30))
    shape = si.ModelShape(f"loop-{seed}", n_layers, n_q * d, n_q, n_kv, d, ffn, vocab, dtype,
                          1e-6 if dtype == "fp32" else 1e-5)
    mask = (rng.random(2 * n_layers) < 0.35).astype(np.uint8)
    max_k = int(rng.integers(1, 32))
    eps = float(rng.choice([0.0, 0.3, 0.8]))
    width = int(rng.choice([1, 3, 10]))
    return shape, max_seq, n_prompt, n_new, mask, max_k, eps, width


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_random_decoding_loops_are_lossless(oracle_lib, dtype):
    """Plain greedy decoding, draft-then-verify decoding and decoding with dynamic verification (Sections 3.1
    and 4.2) on seeded random shapes, masks, draft lengths and thresholds.  fp32 storage: every loop's tokens
    equal the oracle's.  Both storage types: the speculative loops on the GPU reproduce the GPU's own plain
    decoding exactly, so do the oracle's, and the GPU follows the oracle step by step (a token differs only at
    a near tie of the oracle's logits)."""
    import paper_2410_06916_amd as P
    n_done = n_ties = 0
    for seed in range(24):
        shape, max_seq, n_prompt, n_new, mask, max_k, eps, width = _random_loop_case(seed, dtype)
        if shape.hidden % 32:
            continue
        what = (seed, shape, max_seq, n_prompt, n_new, max_k, eps, width)
        weights = hp.shaped_weights(shape, seed=seed)
        o = oracle_lib.Oracle(shape, max_seq, threads=8)
        o.set_weights(weights)
        g = P.SwiftModel(shape, max_seq)
        g.load_weights(weights)
        prompt = si.uniform_ids(2000 + seed, n_prompt, shape.vocab)
        want = oracle_lib.generate_ar(o, prompt, n_new)
        plain = P.generate_ar(g, prompt, n_new)
        w1, _ = oracle_lib.generate_swift(o, prompt, n_new, mask, max_k, eps)
        g1, _ = P.generate_swift(g, prompt, n_new, mask, max_k, eps)
        w2, _ = oracle_lib.generate_swift_tree(o, prompt, n_new, mask, min(max_k, 8), eps, width)
        g2, _ = P.generate_swift_tree(g, prompt, n_new, mask, min(max_k, 8), eps, width)
        assert np.array_equal(w1, want) and np.array_equal(w2, want), what
        assert np.array_equal(g1, plain) and np.array_equal(g2, plain), what
        if dtype == "fp32":
            assert np.array_equal(plain, want), what
        # against the oracle step by step: drafts, stop decisions, verify targets and logits; a token may
        # differ only where the oracle's own top-2 margin is within the tolerance (then the oracle is followed)
        res = hp.lockstep_swift(o, g, prompt, n_new, mask, max_k, eps, TOL[dtype])
        assert np.array_equal(res["tokens"], want), what
        n_ties += sum(res["ties"].values())
        g.close()
        o.close()
        n_done += 1
    assert n_done >= 16
    assert n_ties <= n_done      # near ties are the exception, not the rule
