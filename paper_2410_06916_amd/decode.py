"""Generation loops over the C-ABI calls (host control flow only; every forward pass,
arg-max and confidence runs in the HIP library)."""
from __future__ import annotations

from typing import List, Sequence

import numpy as np


def generate_ar(m, prompt: Sequence[int], n_new: int, want_logits: bool = False):
    """Plain greedy decoding: prefill, then one-row verify + accept per token."""
    out = [m.prefill(prompt)]
    logits = []
    while len(out) < n_new:
        tgt, lg = m.verify([m.pending], want_logits)
        m.accept()
        out.append(int(tgt[0]))
        if want_logits:
            logits.append(lg[0])
    if want_logits:
        return np.array(out, np.int32), logits
    return np.array(out, np.int32)


def generate_swift(m, prompt: Sequence[int], n_new: int, skip: np.ndarray, max_k: int, conf_threshold: float,
                   poison: bool = False, want_logits: bool = False):
    """Draft-then-verify greedy decoding (paper Section 4.2).  The draft length of a step is
    capped at (tokens still wanted - 1), so exactly n_new tokens come out.
    Returns (tokens, trace) with one dict per decoding step."""
    out: List[int] = [m.prefill(prompt)]
    trace: List[dict] = []
    while len(out) < n_new:
        if poison:
            m.poison_kv()
        k_cap = min(max_k, n_new - len(out) - 1)
        n0 = m.cache_len
        if k_cap > 0:
            d, conf = m.draft_step(skip, k_cap, conf_threshold)
        else:
            d, conf = np.zeros(0, np.int32), np.zeros(0, np.float32)
        block = np.concatenate([[m.pending], d]).astype(np.int32)
        tgt, lg = m.verify(block, want_logits)
        em = m.accept()
        out.extend(int(t) for t in em)
        trace.append(dict(n=n0, block=block, draft=d, conf=conf, target=tgt, emitted=em, m=len(em) - 1, logits=lg))
    return np.array(out, np.int32), trace


def generate_swift_tree(m, prompt: Sequence[int], n_new: int, skip: np.ndarray, max_k: int, conf_threshold: float,
                        max_width: int = 10, poison: bool = False, want_logits: bool = False):
    """Draft-then-verify greedy decoding with dynamic verification (paper Section 4.2, both strategies):
    every draft position keeps its top candidates and the token tree is verified in one block.
    Returns (tokens, trace); the last step may emit past n_new, the tokens are cut to n_new."""
    out: List[int] = [m.prefill(prompt)]
    trace: List[dict] = []
    while len(out) < n_new:
        if poison:
            m.poison_kv()
        k_cap = min(max_k, n_new - len(out) - 1)
        n0 = m.cache_len
        if k_cap > 0:
            levels, conf = m.draft_step_topk(skip, k_cap, conf_threshold, max_width)
        else:
            levels, conf = [], np.zeros(0, np.float32)
        tgt, lg = m.verify_tree(levels, want_logits)
        em = m.accept_tree()
        out.extend(int(t) for t in em)
        trace.append(dict(n=n0, levels=levels, conf=conf, target=tgt, emitted=em, m=len(em) - 1, logits=lg))
    return np.array(out[:n_new], np.int32), trace


def generate_swift_on_the_fly(m, opt, prompt: Sequence[int], n_new: int, max_k: int, conf_threshold: float,
                              gamma: int = 32, tree_width: int = 0):
    """The whole method for one input (paper Section 4): prefill; context accumulation with the uniform
    initial pattern until gamma generated tokens are committed (Section 4.1.1); then one optimisation step before
    every decoding step (a candidate from `opt` scored on the last gamma generated tokens, the best one retained
    and used to draft this step, Section 4.1.2) until `opt` terminates; then plain acceleration with the retained
    set (Section 4.2).  tree_width > 0 adds dynamic verification.  Returns (tokens, trace)."""
    out: List[int] = [m.prefill(prompt)]
    mask = opt.initial_mask()
    finished = False
    trace: List[dict] = []
    while len(out) < n_new:
        info = None
        if not finished and len(out) - 1 >= gamma:
            info = opt.step(m, out[-(gamma + 1):])
            mask, finished = info["best"], info["finished"]
        k_cap = min(max_k, n_new - len(out) - 1)
        n0 = m.cache_len
        if tree_width > 0:
            levels = m.draft_step_topk(mask, k_cap, conf_threshold, tree_width)[0] if k_cap > 0 else []
            m.verify_tree(levels)
            em = m.accept_tree()
            n_draft = len(levels)
        else:
            d = m.draft_step(mask, k_cap, conf_threshold)[0] if k_cap > 0 else np.zeros(0, np.int32)
            m.verify(np.concatenate([[m.pending], d]).astype(np.int32))
            em = m.accept()
            n_draft = len(d)
        out.extend(int(t) for t in em)
        trace.append(dict(n=n0, mask=np.array(mask, np.uint8), opt=info, n_draft=n_draft, emitted=em, m=len(em) - 1))
    return np.array(out[:n_new], np.int32), trace


SAMPLE_U_PER_STEP = 31  # uniforms one decoding step may use: 15 draws, 15 acceptance tests, 1 final draw


def generate_swift_sample(m, prompt: Sequence[int], n_new: int, skip: np.ndarray, max_k: int, conf_threshold: float,
                          temperature: float, top_p: float, u0: float, U: np.ndarray, want_probs: bool = False):
    """Draft-then-verify decoding with speculative sampling (paper Section 5.1, Appendix B.2).  The caller
    supplies the uniforms: u0 for the first token, U[s] for decoding step s ([0:15] the draft draws,
    [15:30] the acceptance tests, [30] the final draw).  Returns (tokens, trace)."""
    out: List[int] = [m.prefill_sample(prompt, temperature, top_p, u0)]
    trace: List[dict] = []
    s = 0
    while len(out) < n_new:
        k_cap = min(max_k, n_new - len(out) - 1)
        n0 = m.cache_len
        if k_cap > 0:
            d, conf = m.draft_step_sample(skip, k_cap, conf_threshold, temperature, top_p, U[s, 0:15])
        else:
            d, conf = np.zeros(0, np.int32), np.zeros(0, np.float32)
        block = np.concatenate([[m.pending], d]).astype(np.int32)
        em, pr = m.verify_sample(block, temperature, top_p, U[s, 15:30], float(U[s, 30]), want_probs)
        out.extend(int(t) for t in em)
        trace.append(dict(n=n0, draft=d, conf=conf, emitted=em, m=len(em) - 1, probs=pr))
        s += 1
    return np.array(out[:n_new], np.int32), trace
