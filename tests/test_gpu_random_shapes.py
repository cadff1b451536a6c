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
        o.prefill(prompt)
        g.prefill(prompt)
        if g.pending != o.pending:              # a near tie in the prompt's last row: follow the oracle
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
