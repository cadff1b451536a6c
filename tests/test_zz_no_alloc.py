"""The allocation-free verification entry point (swift_verify_static: the kernels' scratch in a device array
that is part of the library instead of in the caller's arena) against swift_verify, through the C ABI:
same target tokens and the same logits bit for bit -- they are the same kernels -- on two calls in a row,
the second with a smaller block, with data left in the array by the first."""
import numpy as np
import pytest

import synthetic_inputs as si
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _both(g, block):
    """The block through swift_verify and through swift_verify_static from the same state."""
    n0, t0 = g.cache_len, g.pending
    ta, la = g.verify(block, True)
    g.rollback(n0, t0)
    ts, ls = g.verify_static(block, True)
    return (ta, la), (ts, ls)


def test_static_scratch_verify_equals_arena_verify_on_two_calls_in_a_row():
    import paper_2410_06916_amd as P
    # 7B widths, two layers, a cache beyond the short-context attention kernel: a 9-row block splits K over
    # workgroups in three of its projections (partial sums + arrival counters) and its attention over cache
    # ranges (partial results); a 3-row block afterwards uses the attention partials only
    shape = si.LLAMA2_7B.with_layers(2)
    g = P.SwiftModel(shape, 1700)
    for nm, t in si.iter_weights(shape, 0, "cuda:0"):
        g.load_tensor(nm, t)
    g.prefill(si.uniform_ids(4, 300, shape.vocab))
    n0, t0 = g.cache_len, g.pending
    rng = np.random.default_rng(1)
    big = np.concatenate(([t0], rng.integers(0, shape.vocab, 8))).astype(np.int32)
    small = big[:3].copy()
    # reference results from the existing entry point
    ta_big, la_big = g.verify(big, True)
    g.rollback(n0, t0)
    ta_small, la_small = g.verify(small, True)
    g.rollback(n0, t0)
    # two calls in a row through the static array, the second smaller
    ts_big, ls_big = g.verify_static(big, True)
    g.rollback(n0, t0)
    ts_small, ls_small = g.verify_static(small, True)
    assert np.array_equal(ts_big, ta_big) and np.array_equal(ls_big, la_big)
    assert np.array_equal(ts_small, ta_small) and np.array_equal(ls_small, la_small)
    # the state machine goes on as after swift_verify
    em = g.accept()
    assert len(em) >= 1 and g.cache_len == n0 + len(em)
    # and the arena path still gives the same after the static calls
    g.rollback(n0, t0)
    tb, lb = g.verify(big, True)
    assert np.array_equal(tb, ta_big) and np.array_equal(lb, la_big)
    g.close()


def test_static_scratch_verify_against_oracle_and_limits(oracle_lib):
    import paper_2410_06916_amd as P
    # against the oracle, to the bar of every other parity test (tokens exact, logits within the bf16 tolerance)
    shape = hp.SMALL_GQA_BF16
    weights = hp.shaped_weights(shape, seed=21)
    o = oracle_lib.Oracle(shape, 1700, threads=4)
    o.set_weights(weights)
    g = P.SwiftModel(shape, 1700)
    g.load_weights(weights)
    prompt = si.uniform_ids(11, 90, shape.vocab)
    assert g.prefill(prompt) == o.prefill(prompt)[0]
    for k in (11, 4, 0):
        block = np.concatenate(([o.pending], si.uniform_ids(50 + k, k, shape.vocab))).astype(np.int32)
        to, lo = o.verify(block, True)
        tg, lg = g.verify_static(block, True)
        assert np.array_equal(tg, to)
        assert np.all(hp.rel_err_rowmax(lg, lo) <= 2e-2)
        assert np.array_equal(g.accept(), o.accept())
    g.close()
    o.close()
    # a block whose attention partials do not fit the array is refused before anything runs
    wide = si.ModelShape("wide-heads", 1, 256, 64, 8, 128, 256, 512, "bf16", 1e-5)
    g = P.SwiftModel(wide, 4000)
    g.load_weights(si.make_weights(wide, 0))
    t = g.prefill(si.uniform_ids(2, 20, wide.vocab))
    n0 = g.cache_len
    with pytest.raises(P.SwiftError) as e:
        g.verify_static([t] + [1] * 15)
    assert e.value.code == -2 and "static scratch" in str(e.value)
    assert g.cache_len == n0 and g.pending == t
    g.verify_static([t, 1])              # a small block of the same model fits
    g.accept()
    with pytest.raises(P.SwiftError) as e:
        g.verify_static([g.pending, wide.vocab])      # the argument checks are swift_verify's
    assert e.value.code == -1
    g.close()
