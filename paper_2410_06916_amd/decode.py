"""Generation over the C-ABI calls.  Host control flow only: every forward pass, arg-max, confidence,
draw and acceptance test runs in the HIP library.

One driver (`_generate`) owns the token budget; what a decoding step does (plain greedy, draft-then-verify
with a chain or a token tree, speculative sampling, an optimisation step first) is a callable handed to it.
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

# A decoding step: room = tokens still wanted (>= 1) -> (tokens it emitted, a record for the trace).
Step = Callable[[int], Tuple[np.ndarray, dict]]

_NO_TOKENS = np.zeros(0, np.int32)
_NO_CONF = np.zeros(0, np.float32)


def _generate(first_token: int, n_new: int, step: Step) -> Tuple[np.ndarray, List[dict]]:
    """Runs `step` until n_new tokens exist (the first one comes from the prefill).  A step may emit more
    than there is room for only if it ignores `room`; the result is cut to n_new either way."""
    tokens = [int(first_token)]
    trace: List[dict] = []
    while len(tokens) < n_new:
        emitted, record = step(n_new - len(tokens))
        tokens += [int(t) for t in emitted]
        trace.append(record)
    return np.asarray(tokens[:n_new], np.int32), trace


def _draft_budget(max_k: int, room: int) -> int:
    """Draft tokens worth asking for: a verify pass emits at most one token more than it was given drafts."""
    return max(0, min(max_k, room - 1))


def _chain_step(m, skip, max_k: int, conf_threshold: float, poison: bool, want_logits: bool) -> Step:
    """Section 4.2, first strategy: draft with early stopping, verify the chain, accept the matching prefix."""
    def step(room: int):
        if poison:
            m.poison_kv()
        n_before = m.cache_len
        budget = _draft_budget(max_k, room)
        draft, conf = m.draft_step(skip, budget, conf_threshold) if budget else (_NO_TOKENS, _NO_CONF)
        block = np.concatenate(([m.pending], draft)).astype(np.int32)
        target, logits = m.verify(block, want_logits)
        emitted = m.accept()
        return emitted, dict(n=n_before, block=block, draft=draft, conf=conf, target=target, emitted=emitted,
                             m=len(emitted) - 1, logits=logits)
    return step


def _tree_step(m, skip, max_k: int, conf_threshold: float, max_width: int, poison: bool, want_logits: bool) -> Step:
    """Section 4.2, both strategies: every draft position keeps its top candidates; one block verifies the tree."""
    def step(room: int):
        if poison:
            m.poison_kv()
        n_before = m.cache_len
        budget = _draft_budget(max_k, room)
        levels, conf = m.draft_step_topk(skip, budget, conf_threshold, max_width) if budget else ([], _NO_CONF)
        target, logits = m.verify_tree(levels, want_logits)
        emitted = m.accept_tree()
        return emitted, dict(n=n_before, levels=levels, conf=conf, target=target, emitted=emitted,
                             m=len(emitted) - 1, logits=logits)
    return step


def generate_ar(m, prompt: Sequence[int], n_new: int, want_logits: bool = False):
    """Plain greedy decoding: prefill, then one one-row target pass per token."""
    rows = []

    def step(_room: int):
        target, logits = m.verify([m.pending], want_logits)
        m.accept()
        if want_logits:
            rows.append(logits[0])
        return target[:1], {}

    tokens, _ = _generate(m.prefill(prompt), n_new, step)
    return (tokens, rows) if want_logits else tokens


def generate_swift(m, prompt: Sequence[int], n_new: int, skip: np.ndarray, max_k: int, conf_threshold: float,
                   poison: bool = False, want_logits: bool = False):
    """Draft-then-verify greedy decoding (paper Section 4.2).  Exactly n_new tokens come out: a step never
    drafts more than (tokens still wanted - 1).  Returns (tokens, trace), one record per decoding step."""
    return _generate(m.prefill(prompt), n_new, _chain_step(m, skip, max_k, conf_threshold, poison, want_logits))


def generate_swift_tree(m, prompt: Sequence[int], n_new: int, skip: np.ndarray, max_k: int, conf_threshold: float,
                        max_width: int = 10, poison: bool = False, want_logits: bool = False):
    """Draft-then-verify greedy decoding with dynamic verification (paper Section 4.2).  Returns (tokens, trace)."""
    return _generate(m.prefill(prompt), n_new,
                     _tree_step(m, skip, max_k, conf_threshold, max_width, poison, want_logits))


def generate_swift_on_the_fly(m, opt, prompt: Sequence[int], n_new: int, max_k: int, conf_threshold: float,
                              gamma: int = 32, tree_width: int = 0):
    """The whole method for one input (paper Section 4): prefill; context accumulation with the uniform
    initial pattern until gamma generated tokens are committed (Section 4.1.1); then one optimisation step
    before every decoding step -- a candidate from `opt` scored on the last gamma generated tokens, the best
    one retained and used to draft that very step (Section 4.1.2) -- until `opt` terminates; then acceleration
    with the retained set (Section 4.2).  tree_width > 0 adds dynamic verification.  Returns (tokens, trace)."""
    generated: List[int] = [m.prefill(prompt)]       # every emitted token so far (the window is cut from it)
    state = dict(mask=opt.initial_mask(), searching=True)

    def step(room: int):
        info: Optional[dict] = None
        if state["searching"] and len(generated) - 1 >= gamma:
            info = opt.step(m, generated[-(gamma + 1):])
            state["mask"], state["searching"] = info["best"], not info["finished"]
        mask = state["mask"]
        inner = (_tree_step(m, mask, max_k, conf_threshold, tree_width, False, False) if tree_width > 0
                 else _chain_step(m, mask, max_k, conf_threshold, False, False))
        emitted, rec = inner(room)
        generated.extend(int(t) for t in emitted)
        n_draft = len(rec["levels"]) if tree_width > 0 else len(rec["draft"])
        return emitted, dict(n=rec["n"], mask=np.array(mask, np.uint8), opt=info, n_draft=n_draft, emitted=emitted,
                             m=rec["m"])

    return _generate(generated[0], n_new, step)


SAMPLE_DRAWS = 15                        # draft draws (and acceptance tests) one decoding step may use
SAMPLE_U_PER_STEP = 2 * SAMPLE_DRAWS + 1  # ... and one final draw


def generate_swift_sample(m, prompt: Sequence[int], n_new: int, skip: np.ndarray, max_k: int, conf_threshold: float,
                          temperature: float, top_p: float, u0: float, U: np.ndarray, want_probs: bool = False):
    """Draft-then-verify decoding with speculative sampling (paper Section 5.1, Appendix B.2).  The caller
    supplies the uniforms: u0 for the first token, row s of U for decoding step s -- the draft draws first,
    then the acceptance tests, the final draw last.  Returns (tokens, trace)."""
    D = SAMPLE_DRAWS
    steps_done = [0]

    def step(room: int):
        u = U[steps_done[0]]
        steps_done[0] += 1
        n_before = m.cache_len
        budget = _draft_budget(max_k, room)
        draft, conf = (m.draft_step_sample(skip, budget, conf_threshold, temperature, top_p, u[:D]) if budget
                       else (_NO_TOKENS, _NO_CONF))
        block = np.concatenate(([m.pending], draft)).astype(np.int32)
        emitted, probs = m.verify_sample(block, temperature, top_p, u[D:2 * D], float(u[2 * D]), want_probs)
        return emitted, dict(n=n_before, draft=draft, conf=conf, emitted=emitted, m=len(emitted) - 1, probs=probs)

    return _generate(m.prefill_sample(prompt, temperature, top_p, u0), n_new, step)
