"""Test-side input shaping shared by the oracle pins and the GPU parity tests.

Nothing here is the method's arithmetic: these helpers only rescale the drawn
weights so that a random-init model behaves less degenerately (draft and target
sometimes agree, confidences spread over (0,1)), and define a few small shapes.
"""
from __future__ import annotations

import dataclasses
from typing import Dict

import torch

import synthetic_inputs as si

# small shapes: GQA (4 query heads on 2 KV heads), non-square everywhere
SMALL_GQA = si.ModelShape("small-gqa", 3, 96, 4, 2, 16, 136, 200, "fp32", 1e-6)
SMALL_GQA_BF16 = dataclasses.replace(SMALL_GQA, name="small-gqa-bf16", dtype="bf16", rms_eps=1e-5)
ONE_LAYER = si.ModelShape("one-layer", 1, 48, 4, 2, 12, 80, 64, "fp32", 1e-6)


def shaped_weights(shape: si.ModelShape, seed: int = 0, branch_scale: float = 0.15, head_scale: float = 40.0,
                   gain_jitter: float = 0.1, device="cpu") -> Dict[str, torch.Tensor]:
    """Drawn weights with the sublayer output projections (wo, wd) shrunk and the
    LM head enlarged.  Small branches make a layer-skipping draft agree with the
    target often but not always; a large head spreads the top-1 probability over
    (0,1) so that the confidence threshold actually decides something."""
    w = si.make_weights(shape, seed, device, gain_jitter=gain_jitter)
    for name in list(w):
        if name.endswith(".wo") or name.endswith(".wd"):
            w[name] = (w[name].float() * branch_scale).to(w[name].dtype)
        elif name == "lm_head":
            w[name] = (w[name].float() * head_scale).to(w[name].dtype)
    return w


def rel_err_rowmax(a, b):
    """max_i |a_i - b_i| / max_i |b_i| per row (b is the reference)."""
    import numpy as np
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    if a.ndim == 1:
        a, b = a[None], b[None]
    return np.max(np.abs(a - b), axis=-1) / np.max(np.abs(b), axis=-1)


def top2_margin(logits_row) -> float:
    """Gap between the two largest logits of a row, relative to the row's largest magnitude."""
    import numpy as np
    row = np.asarray(logits_row, np.float64)
    top = np.partition(row, -2)[-2:]
    return float((top[1] - top[0]) / np.abs(row).max())


def lockstep_swift(o, g, prompt, n_new, mask, max_k, eps, tol, poison=False):
    """Drives the oracle `o` and the library `g` through prefill and draft -> verify -> accept steps side by
    side.  Token ids must be equal; where one differs (a draft token, a stop decision, a verify target, the
    prefill's token) the oracle's own top-2 margin (or the confidence's distance from the threshold) at that
    position must be within `tol` -- anything larger is a bug, not rounding -- and the run goes on
    teacher-forced with the oracle's token.  Verify logits are compared row by row.  Returns a dict with the
    emitted tokens and how often each kind of near tie occurred."""
    import numpy as np
    ties = dict(prefill=0, draft=0, stop=0, target=0)
    rows_checked = max_rows = decisions = 0
    prompt = np.asarray(prompt, np.int32)
    emitted = []

    def prefill_both(ids, kind):
        to, lo = o.prefill(ids)
        tg = g.prefill(ids)
        if tg != to:
            assert top2_margin(lo) <= tol, (kind, "prefill token differs at a clear margin", top2_margin(lo))
            ties[kind] += 1
            g.rollback(g.cache_len, int(to))
        return int(to)

    emitted.append(prefill_both(prompt, "prefill"))
    while len(emitted) < n_new:
        if poison:
            o.poison_kv()
            g.poison_kv()
        n0, pend = o.cache_len, int(o.pending)
        assert (g.cache_len, g.pending) == (n0, pend)
        budget = max(0, min(max_k, n_new - len(emitted) - 1))
        do = np.zeros(0, np.int32)
        if budget:
            do, co = o.draft_step(mask, budget, eps)
            decisions += len(do)
            dg, cg = g.draft_step(mask, budget, eps)
            common = 0
            while common < min(len(do), len(dg)) and do[common] == dg[common]:
                common += 1
            if common < min(len(do), len(dg)):
                # a draft token differs: the oracle's draft logits at that position must be a near tie
                prev = pend if common == 0 else int(do[common - 1])
                lg = o.forward_row(prev, n0 + common, mask)
                assert top2_margin(lg) <= tol, ("draft token differs at a clear margin", n0, common, top2_margin(lg))
                ties["draft"] += 1
            elif len(do) != len(dg):
                # same tokens, one side stopped earlier: that confidence sits at the threshold
                c = co[common - 1] if len(do) < len(dg) else cg[common - 1]
                assert abs(float(c) - eps) <= 5 * max(tol, 1e-4) * max(eps, 1e-3), ("stop decision differs", n0, float(c), eps)
                ties["stop"] += 1
            if common:
                assert np.allclose(cg[:common], co[:common], rtol=5 * max(tol, 1e-4), atol=1e-7), (n0, cg, co)
        block = np.concatenate(([pend], do)).astype(np.int32)      # teacher-forced: the oracle's drafts
        to, lo = o.verify(block, True)
        tg, lg = g.verify(block, True)
        err = rel_err_rowmax(lg, lo)
        assert np.all(err <= tol), ("verify logits", n0, err.max())
        rows_checked += len(block)
        decisions += len(block)
        max_rows = max(max_rows, len(block))
        em = o.accept()
        if np.array_equal(tg, to):
            assert np.array_equal(g.accept(), em)
            emitted += [int(t) for t in em]
            continue
        for r in np.nonzero(np.asarray(tg) != np.asarray(to))[0]:
            assert top2_margin(lo[r]) <= tol, ("verify target differs at a clear margin", n0, int(r), top2_margin(lo[r]))
            ties["target"] += 1
        emitted += [int(t) for t in em]
        if len(emitted) < n_new:
            # go on from the oracle's sequence: both sides prefill everything but the last emitted token
            ids = np.concatenate((prompt, np.asarray(emitted[:-1], np.int32))).astype(np.int32)
            tok = prefill_both(ids, "target")
            assert tok == emitted[-1]   # (the oracle's block forward is its row forward: same token)
    return dict(tokens=np.asarray(emitted[:n_new], np.int32), ties=ties, rows_checked=rows_checked, max_rows=max_rows,
                decisions=decisions)
