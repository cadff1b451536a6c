"""GPU parity: the HIP library (through its C ABI) against the CPU oracle on the
same seeded inputs.  Token ids, draft lengths and accepted counts must match
exactly; logits within 1e-4 (fp32 storage) / 2e-2 (bf16 storage) of the row's
largest magnitude; confidences to the same relative tolerance."""
import dataclasses

import numpy as np
import pytest
import torch

import synthetic_inputs as si
from tests import helpers as hp

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-4, "bf16": 2e-2}


def _pair(oracle_lib, shape, weights, max_seq, threads=8):
    import paper_2410_06916_amd as P
    o = oracle_lib.Oracle(shape, max_seq, threads=threads)
    o.set_weights(weights)
    g = P.SwiftModel(shape, max_seq)
    g.load_weights(weights)
    return o, g


def _compare_traces(shape, to, tg):
    tol = TOL[shape.dtype]
    assert len(to) == len(tg)
    for so, sg in zip(to, tg):
        assert so["n"] == sg["n"]
        assert np.array_equal(so["draft"], sg["draft"]), (so["draft"], sg["draft"])
        assert np.array_equal(so["target"], sg["target"])
        assert so["m"] == sg["m"] and np.array_equal(so["emitted"], sg["emitted"])
        if len(so["conf"]):
            assert np.allclose(sg["conf"], so["conf"], rtol=max(tol, 1e-4) * 5, atol=1e-7)
        if so["logits"] is not None:
            assert np.all(hp.rel_err_rowmax(sg["logits"], so["logits"]) <= tol)


@pytest.fixture(scope="module")
def tiny(oracle_lib):
    w = si.WORKLOADS["tiny"]
    weights = si.make_weights(w.shape, w.weight_seed)
    o, g = _pair(oracle_lib, w.shape, weights, w.n_prompt + w.n_new + w.max_k + 1)
    yield w, o, g
    g.close()


def test_tiny_workload_autoregressive(oracle_lib, tiny):
    import paper_2410_06916_amd as P
    w, o, g = tiny
    prompt = si.workload_prompt(w)
    want, wl = oracle_lib.generate_ar(o, prompt, w.n_new, want_logits=True)
    got, gl = P.generate_ar(g, prompt, w.n_new, want_logits=True)
    assert np.array_equal(got, want)
    err = hp.rel_err_rowmax(np.stack(gl), wl[1:])
    assert err.max() <= TOL["fp32"], err.max()
    assert g.cache_len == o.cache_len and g.pending == o.pending


@pytest.mark.parametrize("eps", [0.8, 0.0])
def test_tiny_workload_speculative(oracle_lib, tiny, eps):
    import paper_2410_06916_amd as P
    w, o, g = tiny
    prompt = si.workload_prompt(w)
    mask = si.workload_mask(w)
    want, to = oracle_lib.generate_swift(o, prompt, w.n_new, mask, w.max_k, eps, want_logits=True)
    got, tg = P.generate_swift(g, prompt, w.n_new, mask, w.max_k, eps, want_logits=True)
    assert np.array_equal(got, want)
    _compare_traces(w.shape, to, tg)
    so, sg = o.stats(), g.stats()
    assert (sg["draft_passes"], sg["verify_passes"], sg["accepted"], sg["emitted_total"]) == \
           (so["draft_passes"], so["verify_passes"], so["accepted"], so["emitted"])
    assert sg["emitted_by_verify"] == sg["emitted_total"] - 1


@pytest.mark.parametrize("shape", [hp.SMALL_GQA, hp.SMALL_GQA_BF16], ids=lambda s: s.name)
def test_small_gqa_masks_thresholds_and_poison(oracle_lib, shape):
    """Grouped-query shape with shaped weights: partial acceptance and early stops
    really happen; slots beyond the cache length are NaN-filled before every step."""
    import paper_2410_06916_amd as P
    weights = hp.shaped_weights(shape, seed=21)
    o, g = _pair(oracle_lib, shape, weights, 96, threads=1)
    prompt = si.uniform_ids(11, 12, shape.vocab)
    rng = np.random.default_rng(5)
    L2 = 2 * shape.n_layers
    masks = [np.zeros(L2, np.uint8), np.ones(L2, np.uint8)] + [(rng.random(L2) < 0.5).astype(np.uint8)
                                                               for _ in range(4)]
    partial = 0
    for i, mask in enumerate(masks):
        for max_k, eps in ((4, 0.5), (7, 0.0), (15, 0.3)):
            want, to = oracle_lib.generate_swift(o, prompt, 40, mask, max_k, eps, poison=True, want_logits=True)
            got, tg = P.generate_swift(g, prompt, 40, mask, max_k, eps, poison=True, want_logits=True)
            assert np.array_equal(got, want), (i, max_k, eps)
            _compare_traces(shape, to, tg)
            partial += sum(0 < s["m"] < len(s["draft"]) for s in tg)
    assert partial > 0
    g.close()


def test_draft_logits_and_cache_contents(oracle_lib):
    """Draft-pass logits (read back through the debug hook) and the key/value slots a
    draft pass and a verify pass leave behind."""
    shape = hp.SMALL_GQA
    weights = hp.shaped_weights(shape, seed=3)
    o, g = _pair(oracle_lib, shape, weights, 64, threads=1)
    prompt = si.uniform_ids(4, 20, shape.vocab)
    assert g.prefill(prompt) == o.prefill(prompt)[0]
    mask = np.zeros(2 * shape.n_layers, np.uint8)
    mask[2] = 1   # attention of layer 1
    mask[5] = 1   # MLP of layer 2
    do, co = o.draft_step(mask, 1, 0.0)
    dg, cg = g.draft_step(mask, 1, 0.0)
    assert np.array_equal(do, dg)
    want = o.forward_row(int(o.pending), o.cache_len, mask)      # same pass again, same slot
    assert hp.rel_err_rowmax(g.read_logits(0), want)[0] <= 1e-4
    for layer in (0, 2):                                           # non-skipped attention sublayers
        ko, vo = o.read_kv(layer, o.cache_len)
        kg, vg = g.read_kv(layer, g.cache_len)
        assert np.allclose(kg, ko, rtol=1e-5, atol=1e-6) and np.allclose(vg, vo, rtol=1e-5, atol=1e-6)
    block = np.concatenate([[o.pending], do]).astype(np.int32)
    to, _ = o.verify(block)
    tg, _ = g.verify(block)
    assert np.array_equal(to, tg)
    for layer in range(shape.n_layers):                            # verify rewrote every layer's slots
        for pos in (o.cache_len, o.cache_len + 1):
            ko, vo = o.read_kv(layer, pos)
            kg, vg = g.read_kv(layer, pos)
            assert np.allclose(kg, ko, rtol=1e-5, atol=1e-6) and np.allclose(vg, vo, rtol=1e-5, atol=1e-6)
    g.close()


def _check_prefill(oracle_lib, shape, o, g, n_prompt, n_new=6):
    """First token, the cache a prompt leaves behind (bf16 slots: equal up to one rounding step) and the greedy
    continuation, oracle against library."""
    import paper_2410_06916_amd as P
    prompt = si.uniform_ids(30 + n_prompt, n_prompt, shape.vocab)
    want, wl = oracle_lib.generate_ar(o, prompt, n_new, want_logits=True)
    got, gl = P.generate_ar(g, prompt, n_new, want_logits=True)
    # (a near tie in the oracle's logits may go either way: compare up to the first one, which must be one)
    for i in range(n_new):
        if got[i] != want[i]:
            assert hp.top2_margin(wl[i]) <= TOL["bf16"], (n_prompt, i)
            break
    o.prefill(prompt)
    g.prefill(prompt)
    for layer in range(shape.n_layers):
        for pos in sorted({0, n_prompt // 2, max(0, n_prompt - 65), n_prompt - 1}):
            ko, vo = o.read_kv(layer, pos)
            kg, vg = g.read_kv(layer, pos)
            # a value next to a bf16 rounding boundary may land on the other side (one step: 2^-7 of the value);
            # an element that is small because its terms cancel carries the error of terms of the vector's size
            for got_v, want_v in ((kg, ko), (vg, vo)):
                assert np.all(np.abs(got_v - want_v) <= 2.0 ** -7 * np.abs(want_v) + 2.0 ** -10 * np.abs(want_v).max()), \
                    (n_prompt, layer, pos)
            # (blocks of more than 16 rows carry two of the three bf16 terms of an activation: 2^-17)
            assert (kg != ko).mean() < 0.1 and (vg != vo).mean() < 0.1, (n_prompt, layer, pos)


def test_prefill_block_sizes_against_oracle(oracle_lib):
    """Prompt lengths around the prefill block sizes: one row, the LDS-resident kernel's five, the 16-row verify
    variants, a ragged 64-row block, exactly 64; then the macro blocks of the blocked matrix product (sub-blocks
    of 64 rows, two per workgroup tile, eight per sweep over the weights): 64 + 1, an odd number of sub-blocks,
    lengths on either side of 128, 256 and 512, and a second macro block with a one-block tail.  The depth of
    this shape's down projection (136) is not a multiple of the 32-deep k tile."""
    shape = hp.SMALL_GQA_BF16
    weights = hp.shaped_weights(shape, seed=8)
    o, g = _pair(oracle_lib, shape, weights, 640, threads=4)
    for n_prompt in (1, 5, 6, 16, 17, 63, 64, 65, 127, 128, 129, 150, 255, 256, 257, 511, 512, 513, 600):
        _check_prefill(oracle_lib, shape, o, g, n_prompt)
    g.close()


@pytest.mark.parametrize("subs,rgw", [(-1, 0)] + [(s_, r_) for s_ in (2, 3, 8) for r_ in (1, 2, 3, 4, 5, 6)])
def test_prefill_tilings_against_oracle(oracle_lib, subs, rgw):
    """Every tile shape of the blocked matrix product (1..4 row groups per wavefront on two sub-blocks, 1 or 2 on
    one: another ring depth and another share of the copies per wavefront each) and macro blocks of 2, 3 and 8 sub-blocks, against the one
    64-row block per sweep that the same prompts take with subs = -1; heads of 64 (attention on the matrix
    cores inside the macro block), a row count that leaves row groups past the end of every tile height."""
    shape = si.ModelShape("macro-d64", 2, 224, 4, 2, 64, 344, 300, "bf16", 1e-5)
    weights = hp.shaped_weights(shape, seed=21)
    o, g = _pair(oracle_lib, shape, weights, 700, threads=4)
    g.prefill_blocks(subs, rgw)
    for n_prompt in (100, 192, 333, 650):
        _check_prefill(oracle_lib, shape, o, g, n_prompt, n_new=3)
    g.close()


BLOCK_ATTN_SHAPES = {
    # head_dim 64, two query heads per kv head
    "d64-gqa2": si.ModelShape("d64-gqa2", 2, 256, 4, 2, 64, 344, 384, "bf16", 1e-5),
    # head_dim 128, four query heads on one kv head
    "d128-gqa4": si.ModelShape("d128-gqa4", 2, 512, 4, 1, 128, 344, 384, "bf16", 1e-5),
    # head_dim 128, one kv head per query head
    "d128-mha": si.ModelShape("d128-mha", 2, 256, 2, 2, 128, 344, 384, "bf16", 1e-5),
}


@pytest.mark.parametrize("case", sorted(BLOCK_ATTN_SHAPES))
def test_block_attention_on_matrix_cores_against_oracle(oracle_lib, case):
    """Blocks of 17..64 rows over a bf16 cache with heads of 64 or 128 take the matrix-core attention
    kernel (Section 3.1: the rows of a prefill or verify pass form one causal block).  Prompt lengths that
    give ragged blocks, full blocks, a 64-row block followed by one row, and contexts cut into one to five
    cache ranges; checked through what depends on the attention output of every prompt row: the keys and
    values of the second layer, the logits of the next pass, the greedy continuation.  Then the blocks of
    candidate evaluation (Section 4.1.2) over the same cache."""
    import paper_2410_06916_amd as P
    shape = BLOCK_ATTN_SHAPES[case]
    weights = hp.shaped_weights(shape, seed=12)
    o, g = _pair(oracle_lib, shape, weights, 640, threads=8)
    for n_prompt in (17, 33, 63, 64, 65, 129, 200, 600):
        prompt = si.uniform_ids(70 + n_prompt, n_prompt, shape.vocab)
        fo = o.prefill(prompt)[0]
        fg = g.prefill(prompt)
        for pos in sorted({0, 15, 16, n_prompt // 2, n_prompt - 2, n_prompt - 1}):
            ko, vo = o.read_kv(1, pos)
            kg, vg = g.read_kv(1, pos)
            # (a first-layer slot that rounds to the neighbouring bf16 value on one side shifts every later
            # row a little, so single rounding steps are not the bound here: the bf16 tolerance is)
            assert hp.rel_err_rowmax(kg, ko)[0] <= TOL["bf16"] / 2, (case, n_prompt, pos)
            assert hp.rel_err_rowmax(vg, vo)[0] <= TOL["bf16"] / 2, (case, n_prompt, pos)
        to, lo_ = o.verify([o.pending], True)
        tg, lg = g.verify([g.pending], True)
        assert np.all(hp.rel_err_rowmax(lg, lo_) <= TOL["bf16"]), (case, n_prompt)
        top2 = np.sort(lo_[0])[-2:]
        if top2[1] - top2[0] > 1e-3 * np.abs(lo_[0]).max():   # the arg-max is not a near tie
            assert fg == fo and int(tg[0]) == int(to[0]), (case, n_prompt)
    # candidate evaluation over the 600-token cache: blocks of 18..64 rows that reuse the target's cache
    prompt = si.uniform_ids(70 + 600, 600, shape.vocab)
    o.prefill(prompt)
    g.prefill(prompt)
    window_src = np.concatenate([prompt, [o.pending]]).astype(np.int32)
    masks = [np.zeros(4, np.uint8), np.array([0, 1, 0, 0], np.uint8), np.array([0, 0, 1, 1], np.uint8)]
    for gamma in (17, 40, 64):
        for mi, mask in enumerate(masks):
            po, mo, lgo = o.eval_mask(mask, window_src[-(gamma + 1):], want_logits=True)
            pg, mg = g.eval_mask(mask, window_src[-(gamma + 1):])
            # rows whose arg-max is a near tie may differ; everything else must agree
            srt = np.sort(lgo, axis=1)
            clear = (srt[:, -1] - srt[:, -2]) > 1e-3 * np.abs(lgo).max(axis=1)
            assert clear.mean() > 0.8, (case, gamma, mi)
            assert np.array_equal(np.asarray(pg)[clear], np.asarray(po)[clear]), (case, gamma, mi)
            if clear.all():
                assert mg == mo
    g.close()


@pytest.mark.parametrize("blocks", ["macro-block", "64-row-blocks"])
def test_prefill_at_7b_width_against_oracle(oracle_lib, blocks):
    """The 7B workload's widths (hidden 4096, 32 heads of 128, ffn 11008), two layers deep, a 200-token prompt.
    macro-block: one macro block of four sub-blocks (64, 64, 64 and 8 rows) through the blocked matrix product with
    the tiles this shape takes at four sub-blocks (o_proj and down_proj, with few rows, split their depth over
    workgroups) and the macro block's attention in one launch.  64-row-blocks: three 64-row blocks through the block
    kernels (the third one's attention over two cache ranges) and an 8-row tail."""
    shape = si.LLAMA2_7B.with_layers(2)
    weights = si.make_weights(shape, 0)
    o, g = _pair(oracle_lib, shape, weights, 224, threads=16)
    if blocks == "64-row-blocks":
        g.prefill_blocks(-1)
    prompt = si.uniform_ids(9, 200, shape.vocab)
    fo = o.prefill(prompt)[0]
    fg = g.prefill(prompt)
    for pos in (0, 63, 64, 130, 191, 192, 199):
        ko, vo = o.read_kv(1, pos)
        kg, vg = g.read_kv(1, pos)
        assert hp.rel_err_rowmax(kg, ko)[0] <= TOL["bf16"] / 2, pos
        assert hp.rel_err_rowmax(vg, vo)[0] <= TOL["bf16"] / 2, pos
    to, lo_ = o.verify([o.pending], True)
    tg, lg = g.verify([g.pending], True)
    assert np.all(hp.rel_err_rowmax(lg, lo_) <= TOL["bf16"])
    top2 = np.sort(lo_[0])[-2:]
    if top2[1] - top2[0] > 1e-3 * np.abs(lo_[0]).max():
        assert fg == fo and int(tg[0]) == int(to[0])
    g.close()


@pytest.mark.parametrize("case", ["small-gqa", "small-gqa-bf16", "7b-width-2-layers", "7b-width-long-window"])
def test_candidate_evaluation_against_oracle(oracle_lib, case):
    """Section 4.1.2, Eq. 3-4: predictions of candidate draft models over the last gamma generated
    tokens (block pass with the skip mask, target cache reused, nothing written) and the match
    count, for windows of 1..128 tokens (more than 64: two blocks for fp32 models, one macro block of two
    sub-blocks through the blocked matrix product for bf16 models; the long-window case takes that path at
    the 7B width, heads of 128); the decoding state is untouched."""
    import paper_2410_06916_amd as P
    if case.startswith("7b-width"):
        shape = si.LLAMA2_7B.with_layers(2)
        weights = si.make_weights(shape, 0)
        if case == "7b-width-2-layers":
            n_prompt, n_gen, gammas, threads = 10, 24, (1, 5, 17, 32), 8
        else:
            n_prompt, n_gen, gammas, threads = 10, 104, (65, 100), 8
        masks = [np.zeros(4, np.uint8), np.array([0, 1, 1, 0], np.uint8)]
    else:
        shape = hp.SMALL_GQA if case == "small-gqa" else hp.SMALL_GQA_BF16
        weights = hp.shaped_weights(shape, seed=21)
        n_prompt, n_gen, gammas, threads = 12, 140, (1, 4, 6, 16, 32, 64, 65, 100, 128), 1
        rng = np.random.default_rng(2)
        L2 = 2 * shape.n_layers
        masks = [np.zeros(L2, np.uint8), np.ones(L2, np.uint8)] + [(rng.random(L2) < 0.5).astype(np.uint8)
                                                                   for _ in range(3)]
    o, g = _pair(oracle_lib, shape, weights, n_prompt + n_gen + 8, threads=threads)
    prompt = si.uniform_ids(5, n_prompt, shape.vocab)
    want = oracle_lib.generate_ar(o, prompt, n_gen)
    got = P.generate_ar(g, prompt, n_gen)
    assert np.array_equal(got, want)
    seq = np.concatenate([prompt, want]).astype(np.int32)
    n, pend = g.cache_len, g.pending
    for gamma in gammas:
        for mi, mask in enumerate(masks):
            po, mo = o.eval_mask(mask, seq[-(gamma + 1):])
            pg, mg = g.eval_mask(mask, seq[-(gamma + 1):])
            assert np.array_equal(pg, po) and mg == mo, (case, gamma, mi)
            if shape.dtype == "bf16" and gamma > 64:
                # the same window block by block (macro blocks switched off): the same predictions
                g.prefill_blocks(-1)
                pb, mb = g.eval_mask(mask, seq[-(gamma + 1):])
                g.prefill_blocks(0)
                assert np.array_equal(pb, po) and mb == mo, (case, gamma, mi, "64-row blocks")
                if case == "7b-width-long-window":
                    # every tile shape of the blocked matrix product (with two sub-blocks the matrices of few rows
                    # split the depth over workgroups under each of them)
                    for tiling in range(1, 7):
                        g.prefill_blocks(0, tiling)
                        pt, mt = g.eval_mask(mask, seq[-(gamma + 1):])
                        assert np.array_equal(pt, po) and mt == mo, (case, gamma, mi, "tiling", tiling)
                    g.prefill_blocks(0)
            if mi == 0 and gamma + 1 <= n_gen:
                assert mg == gamma      # nothing skipped, window inside the target model's own output
    assert (g.cache_len, g.pending) == (n, pend)
    # decoding goes on as if nothing had happened
    t_o, _ = o.verify([o.pending]); o.accept()
    t_g, _ = g.verify([g.pending]); g.accept()
    assert int(t_o[0]) == int(t_g[0])
    with pytest.raises(P.SwiftError):
        g.eval_mask(masks[0], np.zeros(g.cache_len + 2, np.int32))
    with pytest.raises(P.SwiftError):
        g.eval_mask(masks[0], np.zeros(130, np.int32))      # gamma 129 > 128
    g.close()


def test_optimisation_phase_follows_the_oracle(oracle_lib):
    """Sections 4.1.1-4.1.2, Appendix B.2: optimisation steps interleaved with decoding steps give the
    same candidates, matchness scores, retained sets and termination as the oracle's; the
    random-search stream is the same on both sides; an external suggester can take every beta-th
    step."""
    import paper_2410_06916_amd as P
    shape = hp.SMALL_GQA_BF16
    weights = hp.shaped_weights(shape, seed=21)
    o, g = _pair(oracle_lib, shape, weights, 160, threads=1)
    prompt = si.uniform_ids(5, 12, shape.vocab)
    L2 = 2 * shape.n_layers
    el = np.ones(L2, np.uint8)
    el[0] = el[-1] = 0
    kw = dict(skip_ratio=0.5, max_steps=14, max_stale=9, stop_matchness=0.95, seed=11, eligible=el)
    oo, og = oracle_lib.Optimizer(L2, **kw), P.Optimizer(L2, **kw)
    assert np.array_equal(oo.initial_mask(), og.initial_mask())
    for step in (2, 3, 50, 1000):
        assert np.array_equal(oo.candidate(step), og.candidate(step))
    seq = list(prompt) + [int(o.prefill(prompt)[0])]
    assert g.prefill(prompt) == seq[-1]
    gamma, steps = 16, 0
    while True:
        # context accumulation / decoding step (plain greedy here), then one optimisation step
        to, _ = o.verify([o.pending]); o.accept()
        tg, _ = g.verify([g.pending]); g.accept()
        assert int(to[0]) == int(tg[0])
        seq.append(int(to[0]))
        if len(seq) - len(prompt) <= gamma:
            continue
        window = np.array(seq[-(gamma + 1):], np.int32)
        ro, rg = oo.step(o, window), og.step(g, window)
        steps += 1
        assert np.array_equal(ro["candidate"], rg["candidate"]) and ro["score"] == rg["score"], steps
        assert np.array_equal(ro["best"], rg["best"]) and ro["best_score"] == rg["best_score"]
        assert ro["finished"] == rg["finished"]
        if ro["finished"]:
            break
    assert 1 <= steps <= 14
    with pytest.raises(P.SwiftError):
        og.step(g, window)
    # an external suggester takes steps 2, 4, ...; declining (None) falls back to random search
    og2 = P.Optimizer(L2, skip_ratio=0.5, max_steps=4, max_stale=100, stop_matchness=2.0, seed=11, eligible=el)
    mine = np.zeros(L2, np.uint8)
    mine[1] = 1
    og2.set_suggester(lambda step, best, score: mine if step == 2 else None, 2)
    r1, r2, r3, r4 = (og2.step(g, window) for _ in range(4))
    assert np.array_equal(r1["candidate"], og2.initial_mask()) and np.array_equal(r2["candidate"], mine)
    assert np.array_equal(r3["candidate"], og2.candidate(3)) and np.array_equal(r4["candidate"], og2.candidate(4))
    assert r4["finished"]
    for x in (oo, og, og2):
        x.close()
    g.close()


_ODD_SHAPES = [
    # name, layers, hidden, q heads, kv heads, head dim, ffn, vocab, dtype
    ("mha-d32", 2, 72, 3, 3, 32, 104, 130, "bf16"),          # group 1, nothing a multiple of 32
    ("gqa4-d64", 2, 200, 8, 2, 64, 328, 514, "bf16"),        # group 4
    ("gqa8-d16", 3, 88, 8, 1, 16, 40, 66, "bf16"),           # group 8, one kv head, ffn < hidden
    ("mqa-d128", 1, 264, 2, 1, 128, 520, 1002, "bf16"),      # group 2, head dim 128, one layer
    ("wide-d128", 2, 1032, 8, 8, 128, 2760, 3002, "bf16"),   # > 1024 wide: several k-tiles per slice, ragged
    ("f32-gqa2-d32", 2, 136, 4, 2, 32, 88, 250, "fp32"),     # the storage-generic path
]


@pytest.mark.parametrize("spec", _ODD_SHAPES, ids=[s[0] for s in _ODD_SHAPES])
def test_odd_shapes_against_oracle(oracle_lib, spec):
    """Shapes whose sizes are ragged against every tile (k-tiles of 32, row groups of 16, gate/up
    groups of 8, 64-row prefill blocks) and every grouping of query heads per kv head: prefill of a
    ragged prompt, speculative decoding with a random mask and forced / confidence-stopped drafts,
    candidate evaluation."""
    import paper_2410_06916_amd as P
    name, L, H, nq, nkv, d, F, V, dtype = spec
    shape = si.ModelShape(name, L, H, nq, nkv, d, F, V, dtype, 1e-5 if dtype == "bf16" else 1e-6)
    weights = hp.shaped_weights(shape, seed=len(name))
    n_prompt = 70 if H < 1000 else 23
    o, g = _pair(oracle_lib, shape, weights, n_prompt + 40, threads=4)
    prompt = si.uniform_ids(17, n_prompt, V)
    rng = np.random.default_rng(L * H)
    mask = (rng.random(2 * L) < 0.5).astype(np.uint8)
    for max_k, eps in ((6, 0.0), (15, 0.4)):
        want, to = oracle_lib.generate_swift(o, prompt, 20, mask, max_k, eps, want_logits=True)
        got, tg = P.generate_swift(g, prompt, 20, mask, max_k, eps, want_logits=True)
        assert np.array_equal(got, want), (name, max_k, eps)
        _compare_traces(shape, to, tg)
    seq = np.concatenate([prompt, want]).astype(np.int32)
    # the last run left the final emitted tokens uncommitted or truncated: evaluate inside a fresh AR run
    want = oracle_lib.generate_ar(o, prompt, 20)
    got = P.generate_ar(g, prompt, 20)
    assert np.array_equal(got, want)
    seq = np.concatenate([prompt, want]).astype(np.int32)
    for gamma in (7, 19):
        po, mo = o.eval_mask(mask, seq[-(gamma + 1):])
        pg, mg = g.eval_mask(mask, seq[-(gamma + 1):])
        assert np.array_equal(pg, po) and mg == mo, (name, gamma)
    g.close()


def _compare_tree_traces(shape, to, tg):
    tol = TOL[shape.dtype]
    assert len(to) == len(tg)
    for so, sg in zip(to, tg):
        assert so["n"] == sg["n"]
        assert len(so["levels"]) == len(sg["levels"])
        for lo, lg in zip(so["levels"], sg["levels"]):
            assert np.array_equal(lo, lg), (lo, lg)
        assert np.array_equal(so["target"], sg["target"])
        assert so["m"] == sg["m"] and np.array_equal(so["emitted"], sg["emitted"])
        if len(so["conf"]):
            assert np.allclose(sg["conf"], so["conf"], rtol=max(tol, 1e-4) * 5, atol=1e-7)


_TREE_CASES = {
    # name: (shape, max_seq, n_prompt)
    "small-gqa": (hp.SMALL_GQA, 96, 12),                       # fp32 storage: the row-at-a-time kernels
    "small-gqa-bf16": (hp.SMALL_GQA_BF16, 96, 12),             # tiled kernels, one-workgroup attention
    "small-gqa-bf16-long-cache": (hp.SMALL_GQA_BF16, 1700, 70),  # split attention
    "mha-d32": (si.ModelShape("mha-d32", 2, 72, 3, 3, 32, 104, 130, "bf16", 1e-5), 96, 12),
    "big-vocab": (si.ModelShape("big-vocab", 1, 64, 2, 1, 32, 96, 33002, "bf16", 1e-5), 80, 9),  # > 32 logits per thread
}


@pytest.mark.parametrize("case", list(_TREE_CASES))
def test_dynamic_verification_against_oracle(oracle_lib, case):
    """Section 4.2, second strategy: top-k candidates per draft position by confidence band, the token
    tree verified in one block, acceptance along the tree with the accepted rows' keys/values moved into
    place.  Candidates, widths, targets, emitted tokens, logits and the cache contents afterwards against
    the oracle, with slots beyond the cache length NaN-filled before every step."""
    import paper_2410_06916_amd as P
    shape, max_seq, n_prompt = _TREE_CASES[case]
    weights = hp.shaped_weights(shape, seed=21)
    o, g = _pair(oracle_lib, shape, weights, max_seq, threads=4)
    prompt = si.uniform_ids(11, n_prompt, shape.vocab)
    rng = np.random.default_rng(5)
    L2 = 2 * shape.n_layers
    masks = [np.ones(L2, np.uint8)] + [(rng.random(L2) < 0.5).astype(np.uint8) for _ in range(2)]
    n_new = 30 if shape.vocab < 1000 else 12
    beside = moved = 0
    for i, mask in enumerate(masks):
        for max_k, eps, max_width in ((4, 0.5, 10), (7, 0.0, 3), (15, 0.3, 10), (6, 0.0, 1)):
            want, to = oracle_lib.generate_swift_tree(o, prompt, n_new, mask, max_k, eps, max_width)
            got, tg = P.generate_swift_tree(g, prompt, n_new, mask, max_k, eps, max_width, poison=True)
            assert np.array_equal(got, want), (case, i, max_k, eps, max_width)
            _compare_tree_traces(shape, to, tg)
            assert g.cache_len == o.cache_len and g.pending == o.pending
            for t in tg:
                # steps whose last accepted token was not its level's first candidate / that moved cache slots
                beside += int(t["m"] > 0 and len(t["levels"][t["m"] - 1]) > 1 and
                              t["emitted"][t["m"] - 1] != t["levels"][t["m"] - 1][0])
                moved += int(t["m"] > 1 and len(t["levels"][0]) > 1)
            if max_width == 1:
                assert all(len(l) == 1 for t in tg for l in t["levels"])
            # the compacted cache: every committed slot of every layer
            for layer in range(shape.n_layers):
                for pos in range(n_prompt, g.cache_len):
                    ko, vo = o.read_kv(layer, pos)
                    kg, vg = g.read_kv(layer, pos)
                    tol = 1e-5 if shape.dtype == "fp32" else 1e-2
                    assert np.allclose(kg, ko, rtol=tol, atol=tol) and np.allclose(vg, vo, rtol=tol, atol=tol), \
                        (case, layer, pos)
    assert moved > 0 and (beside > 0 or not case.startswith("small-gqa")), (beside, moved)
    # logits of one tree block
    mask = masks[1]
    assert g.prefill(prompt) == o.prefill(prompt)[0]
    lo, _ = o.draft_step_topk(mask, 6, 0.0, 10)
    lg_, _ = g.draft_step_topk(mask, 6, 0.0, 10)
    assert all(np.array_equal(a, b) for a, b in zip(lo, lg_)) and len(lo) == len(lg_)
    to_, wl = o.verify_tree(o.pending, lo, want_logits=True)
    tg_, gl = g.verify_tree(lg_, want_logits=True)
    assert np.array_equal(to_, tg_)
    assert np.all(hp.rel_err_rowmax(gl, wl) <= TOL[shape.dtype])
    assert np.array_equal(o.accept_tree(), g.accept_tree())
    g.close()


@pytest.mark.parametrize("case", ["small-gqa-bf16", "small-gqa-bf16-long-cache", "7b-width-2-layers", "d128-mha"])
def test_tree_rows_equal_chain_rows_bit_for_bit(case):
    """A row of a token tree gives, bit for bit, the logits the same path gives when it is verified as a
    chain (which in turn equal those of one-token-at-a-time decoding): dynamic verification then cannot
    change the output.  Trees with several wide levels; after acceptance the moved keys/values serve the
    next steps exactly like those a chain would have written."""
    import paper_2410_06916_amd as P
    if case == "7b-width-2-layers":
        shape, weights, max_seq, n_prompt = si.LLAMA2_7B.with_layers(2), None, 64, 20
    elif case == "d128-mha":
        # one kv head per query head and too few heads for the one-workgroup-per-head kernel: the split
        # kernel's one-, two-, three- and four-row instances
        shape = BLOCK_ATTN_SHAPES[case]
        weights, max_seq, n_prompt = hp.shaped_weights(shape, seed=3), 1700, 70
    else:
        shape = hp.SMALL_GQA_BF16
        weights = hp.shaped_weights(shape, seed=3)
        max_seq, n_prompt = (1700, 70) if case.endswith("long-cache") else (96, 12)
    g = P.SwiftModel(shape, max_seq)
    if weights is None:
        for nm, t in _gpu_weights(shape, 0):
            g.load_tensor(nm, t)
    else:
        g.load_weights(weights)
    g.prefill(si.uniform_ids(4, n_prompt, shape.vocab))
    n0, t0 = g.cache_len, g.pending
    rng = np.random.default_rng(8)
    for widths in ((3, 1, 5, 2), (10, 5), (1, 1, 1, 1, 1, 1, 1), (2, 2, 2, 2, 2, 2, 2, 1), (4,), (10, 10, 10, 1),
                   (1,) * 25):
        g.rollback(n0, t0)
        levels = [rng.integers(0, shape.vocab, w).astype(np.int32) for w in widths]
        tgt, lg = g.verify_tree(levels, True)
        row, spine = 1, [t0]
        for j, lv in enumerate(levels):
            for i, tok in enumerate(lv):
                g.rollback(n0, t0)
                ctgt, clg = g.verify(spine + [int(tok)], True)
                assert int(ctgt[-1]) == int(tgt[row + i])
                assert np.array_equal(clg[-1], lg[row + i]), (case, widths, j, i)
            row += len(lv)
            spine.append(int(lv[0]))
    # acceptance on the tree, then plain decoding: same tokens and logits as a chain all the way
    g.rollback(n0, t0)
    ref_toks, ref_rows = [], []
    for _ in range(10):
        tgt, lg = g.verify([g.pending], True)
        g.accept()
        ref_toks.append(int(tgt[0]))
        ref_rows.append(lg[0].copy())
    g.rollback(n0, t0)
    other = lambda t: (t + 1) % shape.vocab
    # level 1: right token second; level 2: right token first; level 3: right token third (ends the path)
    levels = [np.array([other(ref_toks[0]), ref_toks[0]], np.int32), np.array([ref_toks[1]], np.int32),
              np.array([other(ref_toks[2]), other(other(ref_toks[2])), ref_toks[2]], np.int32)]
    g.verify_tree(levels)
    em = g.accept_tree()
    assert [int(t) for t in em] == ref_toks[:1] + [ref_toks[1]]      # a hit beside the first candidate ends the path
    g.rollback(n0, t0)
    levels[0] = levels[0][::-1].copy()
    g.verify_tree(levels)
    em = g.accept_tree()
    assert [int(t) for t in em] == ref_toks[:4] and g.cache_len == n0 + 4
    for i in range(4, 10):
        tgt, lg = g.verify([g.pending], True)
        g.accept()
        assert int(tgt[0]) == ref_toks[i] and np.array_equal(lg[0], ref_rows[i]), (case, i)
    g.close()


def test_errors_and_state_machine_on_device(oracle_lib):
    import paper_2410_06916_amd as P
    shape = hp.SMALL_GQA
    g = P.SwiftModel(shape, 16)
    with pytest.raises(P.SwiftError) as e:
        g.prefill([1, 2, 3])                       # weights not loaded
    assert e.value.code == -3
    g.load_weights(hp.shaped_weights(shape, seed=1))
    with pytest.raises(P.SwiftError) as e:
        g.verify([1])                              # before prefill
    assert e.value.code == -3
    with pytest.raises(P.SwiftError) as e:
        g.prefill(list(range(16)))                 # no room left
    assert e.value.code == -2
    with pytest.raises(P.SwiftError) as e:
        g.prefill([1, 2, shape.vocab])             # id out of range
    assert e.value.code == -1
    for bad in ((-2, 0), (9, 0), (0, -1), (0, 7)):
        with pytest.raises(P.SwiftError) as e:
            g.prefill_blocks(*bad)                 # block count / tile shape out of range
        assert e.value.code == -1
    t = g.prefill([1, 2, 3])
    with pytest.raises(P.SwiftError) as e:
        g.accept()                                 # nothing verified
    assert e.value.code == -3
    with pytest.raises(P.SwiftError) as e:
        g.verify([t + 1 if t + 1 < shape.vocab else 0])   # first row is not the pending token
    assert e.value.code == -1
    with pytest.raises(P.SwiftError) as e:
        g.draft_step(np.zeros(2 * shape.n_layers, np.uint8), 32, 0.5)   # more than SWIFT_MAX_BLOCK - 1 drafts
    assert e.value.code == -1
    n0 = g.cache_len
    with pytest.raises(P.SwiftError) as e:
        g.draft_step(np.zeros(2 * shape.n_layers, np.uint8), 15, 0.5)   # 3 + 15 + 1 > 16 slots
    assert e.value.code == -2
    with pytest.raises(P.SwiftError) as e:
        g.verify([t] * 14)
    assert e.value.code == -2
    assert g.cache_len == n0 and g.pending == t     # state untouched by failed calls
    # a draft step after a verification that was not accepted cancels it (its slots are overwritten)
    g.verify([g.pending])
    g.draft_step(np.ones(2 * shape.n_layers, np.uint8), 2, 0.0)
    with pytest.raises(P.SwiftError) as e:
        g.accept()
    assert e.value.code == -3
    assert g.cache_len == n0 and g.pending == t
    with pytest.raises(ValueError):
        g.draft_step(np.zeros(3, np.uint8), 1, 0.5)            # a mask of the wrong length never reaches the library
    # explicit roll-back: decode two tokens, rewind, decode them again
    a1, _ = g.verify([g.pending]); g.accept()
    a2, _ = g.verify([g.pending]); g.accept()
    g.rollback(n0, t)
    b1, _ = g.verify([g.pending]); g.accept()
    b2, _ = g.verify([g.pending]); g.accept()
    assert (a1[0], a2[0]) == (b1[0], b2[0])
    g.close()


@pytest.mark.parametrize("tree_width", [0, 10])
def test_whole_method_against_oracle(oracle_lib, tree_width):
    """Section 4 end to end (context accumulation, an optimisation step before every decoding step, then
    acceleration; with and without dynamic verification): same tokens, same layer set in every step, same
    candidates, scores and termination as the oracle, and the output equals plain greedy decoding."""
    import paper_2410_06916_amd as P
    shape = hp.SMALL_GQA_BF16
    weights = hp.shaped_weights(shape, seed=21)
    o, g = _pair(oracle_lib, shape, weights, 160, threads=1)
    prompt = si.uniform_ids(5, 12, shape.vocab)
    L2 = 2 * shape.n_layers
    kw = dict(skip_ratio=0.5, max_steps=12, max_stale=8, stop_matchness=0.95, seed=7)
    oo, og = oracle_lib.Optimizer(L2, **kw), P.Optimizer(L2, **kw)
    want, to = oracle_lib.generate_swift_on_the_fly(o, oo, prompt, 90, 6, 0.3, gamma=10, tree_width=tree_width)
    got, tg = P.generate_swift_on_the_fly(g, og, prompt, 90, 6, 0.3, gamma=10, tree_width=tree_width)
    assert np.array_equal(got, want)
    assert np.array_equal(got, P.generate_ar(g, prompt, 90))
    assert len(to) == len(tg)
    n_opt = 0
    for so, sg in zip(to, tg):
        assert so["n"] == sg["n"] and so["n_draft"] == sg["n_draft"] and np.array_equal(so["emitted"], sg["emitted"])
        assert np.array_equal(so["mask"], sg["mask"])
        assert (so["opt"] is None) == (sg["opt"] is None)
        if so["opt"] is not None:
            n_opt += 1
            for k in ("candidate", "best"):
                assert np.array_equal(so["opt"][k], sg["opt"][k])
            assert so["opt"]["score"] == sg["opt"]["score"] and so["opt"]["finished"] == sg["opt"]["finished"]
    assert 1 <= n_opt <= 12 and to[0]["opt"] is None and to[-1]["opt"] is None
    for x in (oo, og):
        x.close()
    g.close()


def test_tree_errors_and_degenerate_trees_on_device(oracle_lib):
    """Error paths and degenerate shapes of the dynamic-verification calls: the oracle and the library reject
    and accept the same things; a tree without levels is one step of plain decoding; a failed call
    leaves the state untouched."""
    import paper_2410_06916_amd as P
    shape = hp.SMALL_GQA
    weights = hp.shaped_weights(shape, seed=1)
    MAXB = P.binding.MAX_BLOCK
    o, g = _pair(oracle_lib, shape, weights, 40 + MAXB, threads=1)
    mask = np.zeros(2 * shape.n_layers, np.uint8)
    with pytest.raises(P.SwiftError) as e:
        g.draft_step_topk(mask, 3, 0.0)                        # before prefill
    assert e.value.code == -3
    prompt = si.uniform_ids(3, 8, shape.vocab)
    t = g.prefill(prompt)
    assert t == o.prefill(prompt)[0]
    with pytest.raises(P.SwiftError) as e:
        g.accept_tree()                                        # nothing verified
    assert e.value.code == -3
    with pytest.raises(oracle_lib.OracleError):
        o.accept_tree()
    for bad in ([np.arange(11)], [np.arange(10)] * 3 + [np.arange(2)], [np.array([], np.int32)],
                [np.array([shape.vocab])]):                    # too wide, too many rows (33), empty level, bad id
        with pytest.raises(P.SwiftError) as e:
            g.verify_tree([np.asarray(b, np.int32) for b in bad])
        assert e.value.code == -1
    with pytest.raises(P.SwiftError) as e:
        g.draft_step_topk(mask, 3, 0.0, 0)                     # max_width < 1
    assert e.value.code == -1
    n0 = g.cache_len
    assert g.pending == t and n0 == 8
    # a tree without levels is one step of plain decoding
    tg, _ = g.verify_tree([])
    to, _ = o.verify_tree(o.pending, [])
    assert np.array_equal(tg, to)
    eg, eo = g.accept_tree(), o.accept_tree()
    assert np.array_equal(eg, eo) and len(eg) == 1 and g.cache_len == n0 + 1
    # a verify in between cancels an outstanding tree, and the other way round
    g.verify_tree([[1, 2]])
    g.verify([g.pending])
    with pytest.raises(P.SwiftError):
        g.accept_tree()
    g.accept()
    g.verify([g.pending])
    g.verify_tree([[3]])
    with pytest.raises(P.SwiftError):
        g.accept()
    g.accept_tree()
    # capacity: the block is narrowed to the cache slots that are left (every row takes one); with none left the
    # call is refused
    cap = 40 + MAXB
    while o.cache_len < g.cache_len:                   # (the oracle catches up with the steps above)
        o.verify([o.pending]); o.accept()
    assert o.pending == g.pending
    while g.cache_len + 4 < cap:
        to, _ = o.verify([o.pending]); o.accept()
        tg, _ = g.verify([g.pending]); g.accept()
        assert int(to[0]) == int(tg[0])
    lo, _ = o.draft_step_topk(mask, 3, 0.0)
    lg, _ = g.draft_step_topk(mask, 3, 0.0)
    assert len(lo) == len(lg) and all(np.array_equal(a, b) for a, b in zip(lo, lg))
    assert 1 + sum(len(l) for l in lg) == cap - g.cache_len == 4
    g.verify_tree(lg)
    g.rollback(g.cache_len, g.pending)
    while g.cache_len < cap:
        g.verify([g.pending]); g.accept()
    with pytest.raises(P.SwiftError) as e:
        g.draft_step_topk(mask, 3, 0.0)
    assert e.value.code == -2
    g.close()


@pytest.mark.parametrize("base,n_layers", [(si.LLAMA2_7B, 2)], ids=["7b-width-2-layers"])
def test_full_width_narrow_depth(oracle_lib, base, n_layers):
    """Same widths, heads, FFN, vocab and dtype as the 7B workload, two layers deep."""
    import paper_2410_06916_amd as P
    shape = base.with_layers(n_layers)
    weights = si.make_weights(shape, 0)
    o, g = _pair(oracle_lib, shape, weights, 48, threads=8)
    prompt = si.uniform_ids(1, 12, shape.vocab)
    mask = np.array([0, 1, 1, 0], np.uint8)
    want, to = oracle_lib.generate_swift(o, prompt, 10, mask, 3, 0.0, want_logits=True)
    got, tg = P.generate_swift(g, prompt, 10, mask, 3, 0.0, want_logits=True)
    assert np.array_equal(got, want)
    _compare_traces(shape, to, tg)
    g.close()


def test_paper_maximum_draft_length_at_7b_width(oracle_lib):
    """Appendix B.2 sets the maximum draft length to 25: forced-length drafting of 25 tokens and 26-row verify
    blocks at the 7B widths (two layers), step by step against the oracle, and the output equals the library's
    own plain greedy decoding."""
    import paper_2410_06916_amd as P
    shape = si.LLAMA2_7B.with_layers(2)
    g = P.SwiftModel(shape, 160)
    o = oracle_lib.Oracle(shape, 160, threads=16)
    for name, t in _gpu_weights(shape, 0):
        g.load_tensor(name, t)
        o.set_tensor(name, t.cpu())
    prompt = si.uniform_ids(3, 40, shape.vocab)
    mask = np.array([0, 1, 0, 0], np.uint8)
    res = hp.lockstep_swift(o, g, prompt, 60, mask, 25, 0.0, TOL["bf16"])
    # (random-init logits are nearly flat: with bf16 keys and values a few per cent of the arg-max decisions are
    # near ties that may fall either way; each one was checked against the oracle's own margin)
    assert res["max_rows"] == 26 and sum(res["ties"].values()) <= max(2, 0.05 * res["decisions"]), res
    ar = P.generate_ar(g, prompt, 60)
    out, trace = P.generate_swift(g, prompt, 60, mask, 25, 0.0)
    assert np.array_equal(out, ar) and max(len(t["block"]) for t in trace) == 26
    if sum(res["ties"].values()) == 0:
        assert np.array_equal(out, res["tokens"])
    g.close()
    o.close()


_WIDTHS = {"13b": si.LLAMA2_13B, "70b": si.LLAMA2_70B}


@pytest.mark.parametrize("width", ["13b", "70b"])
@pytest.mark.parametrize("scenario", ["short-cache", "long-cache"])
def test_other_widths_narrow_depth_against_oracle(oracle_lib, width, scenario):
    """The 13B and the 70B (64 query heads on 8 kv heads) workloads' widths, heads, FFN, vocabulary and dtype,
    two layers deep, against the oracle step by step (Section 4.2, Eq. 5): drafts, stop decisions, verify
    targets exact -- a differing token must be a near tie of the oracle's own logits -- and every verify row's
    logits within the bf16 tolerance.  short-cache: 12-token prompt, drafts of up to 3 tokens, the attention
    sublayer of layer 1 and the MLP of layer 0 skipped.  long-cache: a cache capacity beyond the short-context
    attention kernel's, a 70-token prompt (one macro block of two sub-blocks, 64 and 6 rows, through the blocked
    matrix product at these widths), drafts of up to 12 tokens
    (13-row verify blocks), both sublayers of layer 0 skipped."""
    import paper_2410_06916_amd as P
    shape = _WIDTHS[width].with_layers(2)
    if scenario == "short-cache":
        max_seq, n_prompt, n_new, mask, max_k = 48, 12, 10, np.array([0, 1, 1, 0], np.uint8), 3
    else:
        max_seq, n_prompt, n_new, mask, max_k = 1700, 70, 15, np.array([1, 1, 0, 0], np.uint8), 12
    g = P.SwiftModel(shape, max_seq)
    o = oracle_lib.Oracle(shape, max_seq, threads=16)
    for name, t in _gpu_weights(shape, 0):
        g.load_tensor(name, t)
        o.set_tensor(name, t.cpu())
    prompt = si.uniform_ids(1, n_prompt, shape.vocab)
    res = hp.lockstep_swift(o, g, prompt, n_new, mask, max_k, 0.0, TOL["bf16"])
    assert len(res["tokens"]) == n_new and res["rows_checked"] >= n_new
    # with forced-length drafts the verify blocks really had max_k + 1 rows
    assert res["max_rows"] == max_k + 1
    assert sum(res["ties"].values()) <= max(2, 0.05 * res["decisions"]), res["ties"]
    g.close()
    o.close()


# attention kernel instance per block size that each case of the bit-for-bit test is meant to reach
_MFMA_7B = "mfma<d 128, group 1, 8 wavefronts, range 256, tiles %d>"     # one workgroup per kv head, no second launch
_MFMA_LONG = "mfma<d 128, group 1, 4 wavefronts, range 128, tiles %d>"   # the cache cut into ranges + merge launch
_EXPECTED_ATTN_PATHS = {
    # heads of 16: the row-at-a-time kernels (vector arithmetic), rows sharing loads two by two
    "small-gqa-bf16": {1: "split<bf16, group 2, rows 1>", 2: "split<bf16, group 2, rows 2>",
                       16: "split<bf16, group 2, rows 2>"},
    "small-gqa-bf16-long-cache": {1: "split<bf16, group 2, rows 1>", 9: "split<bf16, group 2, rows 2>"},
    # heads of 128: the matrix-core kernel, every row of the block a column of one tile
    "7b-width-2-layers": {1: _MFMA_7B % 1, 5: _MFMA_7B % 1, 9: _MFMA_7B % 1, 16: _MFMA_7B % 1, 26: _MFMA_7B % 2},
    "d128-mha": {1: _MFMA_LONG % 1, 2: _MFMA_LONG % 1, 3: _MFMA_LONG % 1, 16: _MFMA_LONG % 1, 32: _MFMA_LONG % 2},
}


@pytest.mark.parametrize("case", ["small-gqa-bf16", "small-gqa-bf16-long-cache", "7b-width-2-layers", "d128-mha"])
def test_block_rows_equal_single_rows_bit_for_bit(case):
    """What makes speculative output equal plain greedy output exactly rather than up to rounding
    (Sections 1 and 3.1: verification leaves the output unchanged): the logits of a token do not
    depend on how many rows share its pass.  Rows of verify blocks of 2..32 tokens against the same
    tokens decoded one at a time, compared bit for bit; both attention kernels, the LDS-resident and
    the block projection kernel, split K over 1..8 workgroups."""
    import paper_2410_06916_amd as P
    if case == "7b-width-2-layers":
        shape, weights, max_seq, n_prompt = si.LLAMA2_7B.with_layers(2), None, 64, 20
    elif case == "d128-mha":
        # heads of 128, one kv head per query head, a cache beyond the short-context kernel's capacity
        shape = BLOCK_ATTN_SHAPES[case]
        weights, max_seq, n_prompt = hp.shaped_weights(shape, seed=3), 1700, 70
    else:
        shape = hp.SMALL_GQA_BF16
        weights = hp.shaped_weights(shape, seed=3)
        max_seq, n_prompt = (1700, 70) if case.endswith("long-cache") else (96, 12)
    g = P.SwiftModel(shape, max_seq)
    # the attention kernel each block size takes is the one the case is meant to cover
    want_path = _EXPECTED_ATTN_PATHS[case]
    for R, name in want_path.items():
        assert g.attn_path(R) == name, (case, R, g.attn_path(R))
    if weights is None:
        for nm, t in _gpu_weights(shape, 0):
            g.load_tensor(nm, t)
    else:
        g.load_weights(weights)
    g.prefill(si.uniform_ids(4, n_prompt, shape.vocab))
    n0, t0 = g.cache_len, g.pending
    toks, rows = [t0], []
    for _ in range(32):
        tgt, lg = g.verify([g.pending], True)
        g.accept()
        toks.append(int(tgt[0]))
        rows.append(lg[0].copy())
    for R in (2, 3, 5, 6, 9, 16, 17, 26, 32):
        g.rollback(n0, t0)
        tgt, lg = g.verify(toks[:R], True)
        assert [int(x) for x in tgt] == toks[1:R + 1]
        for r in range(R):
            assert np.array_equal(lg[r], rows[r]), (case, R, r, np.abs(lg[r] - rows[r]).max())
    g.close()


def test_long_context_uses_split_attention(oracle_lib):
    """A context beyond the single-workgroup attention range (1536 slots): the split kernel and
    its merge, for one row and for a block, with a ragged last chunk."""
    import paper_2410_06916_amd as P
    shape = dataclasses.replace(hp.SMALL_GQA_BF16, name="small-gqa-bf16-long", n_layers=2)
    weights = hp.shaped_weights(shape, seed=33)
    n_prompt = 1601
    o, g = _pair(oracle_lib, shape, weights, n_prompt + 40, threads=8)
    prompt = si.uniform_ids(9, n_prompt, shape.vocab)
    mask = np.array([0, 1, 0, 0], np.uint8)
    want, to = oracle_lib.generate_swift(o, prompt, 12, mask, 5, 0.0, want_logits=True)
    got, tg = P.generate_swift(g, prompt, 12, mask, 5, 0.0, want_logits=True)
    assert np.array_equal(got, want)
    _compare_traces(shape, to, tg)
    g.close()


def _gpu_weights(shape, seed=0):
    """Weights drawn on the GPU (fast at full size); the same tensors feed both sides."""
    return si.iter_weights(shape, seed, "cuda:0")


def test_7b_full_depth_against_oracle(oracle_lib):
    """The full 32-layer 7B shape, in the launch configuration bench.py times, on an input the
    oracle can still afford: short prompt, a few forced-length decoding steps with the workload's
    own skip mask (one-row drafts, a 4-row verify block, 16-row and ragged prefill blocks)."""
    import paper_2410_06916_amd as P
    w = si.WORKLOADS["7b"]
    shape = w.shape
    g = P.SwiftModel(shape, 96)
    o = oracle_lib.Oracle(shape, 96, threads=16)
    for name, t in _gpu_weights(shape, w.weight_seed):
        g.load_tensor(name, t)
        o.set_tensor(name, t.cpu())
    prompt = si.uniform_ids(w.prompt_seed, 21, shape.vocab)
    mask = si.workload_mask(w)
    want, to = oracle_lib.generate_swift(o, prompt, 5, mask, 3, 0.0, want_logits=True)
    got, tg = P.generate_swift(g, prompt, 5, mask, 3, 0.0, want_logits=True)
    assert np.array_equal(got, want)
    _compare_traces(shape, to, tg)
    g.close()


@pytest.mark.parametrize("name,n_prompt,n_new", [("7b", 512, 256), ("13b", 1024, 48), ("7b-long", 8192, 24),
                                                  ("70b", 160, 12)])
def test_full_size_workloads_are_lossless_on_gpu(name, n_prompt, n_new):
    """At the workloads' full shapes (where the oracle is out of reach) the property that holds at
    any size: plain greedy decoding, as-configured speculation and forced-length speculation emit
    the same tokens (Sections 1, 3.1: verification leaves the output unchanged), and the counters
    add up."""
    import paper_2410_06916_amd as P
    w = si.WORKLOADS[name]
    shape = w.shape
    g = P.SwiftModel(shape, n_prompt + n_new + w.max_k + 8)
    for nm, t in _gpu_weights(shape, w.weight_seed):
        g.load_tensor(nm, t)
    prompt = si.uniform_ids(w.prompt_seed, n_prompt, shape.vocab)
    mask = si.workload_mask(w)
    ar = P.generate_ar(g, prompt, n_new)
    assert ar.min() >= 0 and ar.max() < shape.vocab
    for eps, max_k in ((w.conf_threshold, w.max_k), (0.0, w.max_k), (0.0, 15)):
        out, trace = P.generate_swift(g, prompt, n_new, mask, max_k, eps)
        assert np.array_equal(out, ar), (name, eps, max_k)
        st = g.stats()
        assert st["emitted_total"] == n_new and st["verify_passes"] == len(trace)
        assert st["accepted"] == sum(t["m"] for t in trace)
        assert 1 + sum(t["m"] + 1 for t in trace) == n_new
    # dynamic verification: candidate trees instead of chains
    out, trace = P.generate_swift_tree(g, prompt, n_new, mask, w.max_k, w.conf_threshold)
    assert np.array_equal(out, ar), (name, "tree")
    assert 1 + sum(t["m"] + 1 for t in trace) == n_new
    # the whole method: optimisation steps between the decoding steps (random weights: no candidate scores)
    el = np.zeros(mask.size, np.uint8)
    el[4:-4] = 1
    opt = P.Optimizer(mask.size, skip_ratio=0.5, max_steps=6, max_stale=300, stop_matchness=0.95, seed=1, eligible=el)
    out, trace = P.generate_swift_on_the_fly(g, opt, prompt, n_new, w.max_k, w.conf_threshold, gamma=min(32, n_new // 3))
    opt.close()
    assert np.array_equal(out, ar), (name, "on the fly")
    assert 1 <= sum(t["opt"] is not None for t in trace) <= 6
    # no-skip mask: the draft model is the target model, every draft is accepted
    out, trace = P.generate_swift(g, prompt, n_new, np.zeros_like(mask), w.max_k, 0.0)
    assert np.array_equal(out, ar) and all(t["m"] == len(t["draft"]) for t in trace)
    g.close()
