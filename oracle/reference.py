"""ctypes front end of the CPU oracle (oracle/swift_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module,
and this module never imports the product package.

The generation loops below follow the paper's acceleration phase (Section 4.2)
one decoding step at a time: draft -> verify -> accept, with the target model's
plain greedy loop beside it as the definition the method has to reproduce.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "swift_oracle.c")
_LIB = os.path.join(_HERE, "libswift_oracle.so")

F32, BF16 = 0, 1
MAX_BLOCK = 64


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No fast-math and no FMA contraction, so the
    summation order written in the source is the order executed."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                               "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn",
                                          "vocab", "max_seq")] + \
               [("rms_eps", C.c_double), ("rope_theta", C.c_double), ("kv_dtype", C.c_int32)]


_lib = None


class OptConfig(C.Structure):
    _fields_ = [("n_sublayers", C.c_int), ("skip_ratio", C.c_double), ("max_steps", C.c_int), ("max_stale", C.c_int),
                ("stop_matchness", C.c_double), ("seed", C.c_uint64)]


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        vp, i32p, f64p, u8p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_double), C.POINTER(C.c_uint8)
        L.ora_create.argtypes = [C.POINTER(_Config), C.POINTER(vp)]
        L.ora_destroy.argtypes = [vp]
        L.ora_destroy.restype = None
        L.ora_set_threads.argtypes = [vp, C.c_int]
        L.ora_set_threads.restype = None
        L.ora_set_tensor.argtypes = [vp, C.c_char_p, vp, C.c_int, C.c_int64]
        L.ora_forward_row.argtypes = [vp, C.c_int32, C.c_int, u8p, f64p]
        L.ora_eval_mask.argtypes = [vp, u8p, i32p, C.c_int, i32p, C.POINTER(C.c_int), f64p]
        L.ora_topk_width.argtypes = [C.c_double]
        L.ora_topk_width.restype = C.c_int
        L.ora_topk.argtypes = [f64p, C.c_int, C.c_int, i32p]
        L.ora_topk.restype = None
        L.ora_draft_step_topk.argtypes = [vp, u8p, C.c_int, C.c_double, C.c_int, i32p, f64p, C.POINTER(C.c_int),
                                          C.POINTER(C.c_int)]
        L.ora_verify_tree.argtypes = [vp, i32p, C.POINTER(C.c_int), C.c_int, i32p, f64p]
        L.ora_accept_tree.argtypes = [vp, i32p, C.POINTER(C.c_int)]
        L.ora_warp.argtypes = [f64p, C.c_int, C.c_double, C.c_double, f64p, f64p]
        L.ora_warp.restype = None
        L.ora_sample.argtypes = [f64p, C.c_int, C.c_double, f64p]
        L.ora_spec_keep.argtypes = [C.c_double, C.c_double, C.c_double, f64p]
        L.ora_spec_resample.argtypes = [f64p, f64p, C.c_int, C.c_double, f64p]
        L.ora_spec_first_token_batch.argtypes = [f64p, f64p, C.c_int, f64p, C.c_int64, i32p]
        L.ora_spec_first_token_batch.restype = None
        L.ora_prefill_sample.argtypes = [vp, i32p, C.c_int, C.c_double, C.c_double, C.c_double, i32p, f64p]
        L.ora_draft_step_sample.argtypes = [vp, u8p, C.c_int, C.c_double, C.c_double, C.c_double, f64p, i32p, f64p,
                                            C.POINTER(C.c_int), f64p]
        L.ora_verify_sample.argtypes = [vp, i32p, C.c_int, C.c_double, C.c_double, f64p, C.c_double, i32p,
                                        C.POINTER(C.c_int), f64p, f64p]
        L.ora_opt_create.argtypes = [C.POINTER(OptConfig), u8p, C.POINTER(vp)]
        L.ora_opt_destroy.argtypes = [vp]
        L.ora_opt_destroy.restype = None
        L.ora_opt_initial_mask.argtypes = [vp, u8p]
        L.ora_opt_initial_mask.restype = None
        L.ora_opt_candidate.argtypes = [vp, C.c_int, u8p]
        L.ora_opt_candidate.restype = None
        L.ora_opt_step.argtypes = [vp, vp, i32p, C.c_int, u8p, f64p, u8p, f64p, C.POINTER(C.c_int)]
        L.ora_forward_nocache.argtypes = [vp, i32p, C.c_int, f64p]
        L.ora_reset.argtypes = [vp]
        L.ora_prefill.argtypes = [vp, i32p, C.c_int, i32p, f64p]
        L.ora_draft_step.argtypes = [vp, u8p, C.c_int, C.c_double, i32p, f64p, C.POINTER(C.c_int)]
        L.ora_verify.argtypes = [vp, i32p, C.c_int, i32p, f64p]
        L.ora_accept.argtypes = [vp, i32p, C.POINTER(C.c_int)]
        L.ora_rollback.argtypes = [vp, C.c_int, C.c_int32]
        L.ora_cache_len.argtypes = [vp]
        L.ora_pending.argtypes = [vp]
        L.ora_get_stats.argtypes = [vp, C.POINTER(C.c_int64)]
        L.ora_get_stats.restype = None
        L.ora_poison_kv.argtypes = [vp]
        L.ora_poison_kv.restype = None
        L.ora_read_kv.argtypes = [vp, C.c_int, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_float)]
        L.ora_read_kv.restype = None
        L.ora_rmsnorm.argtypes = [f64p, f64p, C.c_int, C.c_double, f64p]
        L.ora_rmsnorm.restype = None
        L.ora_rope.argtypes = [f64p, C.c_int, C.c_int, C.c_double]
        L.ora_rope.restype = None
        L.ora_attend.argtypes = [f64p, C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_int64, C.c_int, C.c_int, f64p]
        L.ora_attend.restype = None
        L.ora_swiglu.argtypes = [C.c_double, C.c_double]
        L.ora_swiglu.restype = C.c_double
        L.ora_argmax_conf.argtypes = [f64p, C.c_int, i32p, f64p]
        L.ora_argmax_conf.restype = None
        L.ora_expected_speedup.argtypes = [C.c_double] * 3
        L.ora_expected_speedup.restype = C.c_double
        L.ora_match_prefix.argtypes = [i32p, i32p, C.c_int]
        L.ora_threads_available.restype = C.c_int
        _lib = L
    return _lib


def _p(a: np.ndarray, ty):
    return a.ctypes.data_as(C.POINTER(ty))


class OracleError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: oracle status {code}")
        self.code = code


def _chk(rc: int, what: str):
    if rc != 0:
        raise OracleError(rc, what)


# ---- free functions (used by the pins) -------------------------------------
def rmsnorm(x, g, eps):
    x = np.ascontiguousarray(x, np.float64)
    g = np.ascontiguousarray(g, np.float64)
    out = np.empty_like(x)
    lib().ora_rmsnorm(_p(x, C.c_double), _p(g, C.c_double), x.size, eps, _p(out, C.c_double))
    return out


def warp(logits, temperature, top_p):
    """(probabilities, margin) of the distribution tokens are sampled from."""
    lg = np.ascontiguousarray(logits, np.float64)
    out = np.empty_like(lg)
    mg = C.c_double()
    lib().ora_warp(_p(lg, C.c_double), lg.size, temperature, top_p, _p(out, C.c_double), C.byref(mg))
    return out, mg.value


def sample(weights, u):
    w = np.ascontiguousarray(weights, np.float64)
    mg = C.c_double()
    return lib().ora_sample(_p(w, C.c_double), w.size, u, C.byref(mg)), mg.value


def spec_keep(p_x, q_x, u):
    return bool(lib().ora_spec_keep(p_x, q_x, u, None))


def spec_resample(p, q, u):
    p = np.ascontiguousarray(p, np.float64)
    q = np.ascontiguousarray(q, np.float64)
    return lib().ora_spec_resample(_p(p, C.c_double), _p(q, C.c_double), p.size, u, None)


def spec_first_token_batch(p, q, u):
    p = np.ascontiguousarray(p, np.float64)
    q = np.ascontiguousarray(q, np.float64)
    u = np.ascontiguousarray(u, np.float64).reshape(-1, 3)
    out = np.empty(u.shape[0], np.int32)
    lib().ora_spec_first_token_batch(_p(p, C.c_double), _p(q, C.c_double), p.size, _p(u, C.c_double), u.shape[0],
                                     _p(out, C.c_int32))
    return out


def rope(v, pos, theta):
    v = np.array(v, np.float64)
    lib().ora_rope(_p(v, C.c_double), v.size, pos, theta)
    return v


def attend(q, k, v):
    """q [d]; k, v [n_ctx][d] float32 -> out [d] float64."""
    q = np.ascontiguousarray(q, np.float64)
    k = np.ascontiguousarray(k, np.float32)
    v = np.ascontiguousarray(v, np.float32)
    out = np.empty(q.size, np.float64)
    lib().ora_attend(_p(q, C.c_double), _p(k, C.c_float), _p(v, C.c_float), k.shape[1], k.shape[0], q.size,
                     _p(out, C.c_double))
    return out


def swiglu(g, u):
    return lib().ora_swiglu(float(g), float(u))


def argmax_conf(logits):
    lg = np.ascontiguousarray(logits, np.float64)
    tok, conf = C.c_int32(), C.c_double()
    lib().ora_argmax_conf(_p(lg, C.c_double), lg.size, C.byref(tok), C.byref(conf))
    return tok.value, conf.value


def expected_speedup(M, alpha, c):
    return lib().ora_expected_speedup(float(M), float(alpha), float(c))


def match_prefix(draft: Sequence[int], target: Sequence[int]) -> int:
    d = np.asarray(draft, np.int32)
    t = np.asarray(target, np.int32)
    return lib().ora_match_prefix(_p(d, C.c_int32), _p(t, C.c_int32), d.size)


def threads_available() -> int:
    return lib().ora_threads_available()


# ---- model -----------------------------------------------------------------
class Optimizer:
    """Optimisation-phase bookkeeping of the oracle (Section 4.1, Appendix B.2): uniform initial
    pattern, random-search candidates under a fixed skip ratio, best candidate retained,
    termination rules."""

    def __init__(self, n_sublayers: int, skip_ratio: float, max_steps: int = 1000, max_stale: int = 300,
                 stop_matchness: float = 0.95, seed: int = 0, eligible: Optional[np.ndarray] = None):
        self.n = n_sublayers
        cfg = OptConfig(n_sublayers, skip_ratio, max_steps, max_stale, stop_matchness, seed)
        el = None if eligible is None else np.ascontiguousarray(eligible, np.uint8)
        h = C.c_void_p()
        _chk(lib().ora_opt_create(C.byref(cfg), None if el is None else _p(el, C.c_uint8), C.byref(h)), "ora_opt_create")
        self._h = h

    def close(self):
        if self._h:
            lib().ora_opt_destroy(self._h)
            self._h = None

    def initial_mask(self) -> np.ndarray:
        m = np.zeros(self.n, np.uint8)
        lib().ora_opt_initial_mask(self._h, _p(m, C.c_uint8))
        return m

    def candidate(self, step: int) -> np.ndarray:
        m = np.zeros(self.n, np.uint8)
        lib().ora_opt_candidate(self._h, step, _p(m, C.c_uint8))
        return m

    def step(self, oracle: "Oracle", window: Sequence[int]):
        """One optimisation step on the window (last gamma committed tokens + pending token).
        Returns dict(candidate, score, best, best_score, finished)."""
        w = np.ascontiguousarray(window, np.int32)
        cand = np.zeros(self.n, np.uint8)
        best = np.zeros(self.n, np.uint8)
        cs, bs, fin = C.c_double(), C.c_double(), C.c_int()
        _chk(lib().ora_opt_step(oracle._h, self._h, _p(w, C.c_int32), w.size - 1, _p(cand, C.c_uint8), C.byref(cs),
                                _p(best, C.c_uint8), C.byref(bs), C.byref(fin)), "ora_opt_step")
        return dict(candidate=cand, score=cs.value, best=best, best_score=bs.value, finished=bool(fin.value))


class Oracle:
    """One model instance + decoding state.  `shape` is any object with the
    attributes n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab,
    rms_eps, rope_theta, dtype ("fp32" | "bf16")."""

    def __init__(self, shape, max_seq: int, threads: int = 1):
        self.shape = shape
        self.vocab = shape.vocab
        cfg = _Config(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                      shape.vocab, max_seq, shape.rms_eps, shape.rope_theta, F32 if shape.dtype == "fp32" else BF16)
        self._h = C.c_void_p()
        _chk(lib().ora_create(C.byref(cfg), C.byref(self._h)), "ora_create")
        lib().ora_set_threads(self._h, threads)
        self._keep: Dict[str, object] = {}

    def close(self):
        if self._h:
            lib().ora_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_threads(self, t: int):
        lib().ora_set_threads(self._h, t)

    def set_tensor(self, name: str, t):
        """t: torch CPU tensor, float32 or bfloat16, contiguous (borrowed, kept alive here)."""
        import torch
        t = t.detach().contiguous()
        assert t.device.type == "cpu"
        if t.dtype == torch.float32:
            dt = F32
        elif t.dtype == torch.bfloat16:
            dt = BF16
        else:
            raise TypeError(t.dtype)
        self._keep[name] = t
        _chk(lib().ora_set_tensor(self._h, name.encode(), C.c_void_p(t.data_ptr()), dt, t.numel()),
             f"ora_set_tensor({name})")

    def set_weights(self, weights):
        for name, t in (weights.items() if hasattr(weights, "items") else weights):
            self.set_tensor(name, t)

    # -- raw forwards
    def forward_row(self, token: int, pos: int, skip: Optional[np.ndarray] = None) -> np.ndarray:
        lg = np.empty(self.vocab, np.float64)
        sp = None
        if skip is not None:
            skip = np.ascontiguousarray(skip, np.uint8)
            sp = _p(skip, C.c_uint8)
        _chk(lib().ora_forward_row(self._h, int(token), int(pos), sp, _p(lg, C.c_double)), "ora_forward_row")
        return lg

    def forward_nocache(self, tokens: Sequence[int]) -> np.ndarray:
        t = np.ascontiguousarray(tokens, np.int32)
        lg = np.empty(self.vocab, np.float64)
        _chk(lib().ora_forward_nocache(self._h, _p(t, C.c_int32), t.size, _p(lg, C.c_double)), "ora_forward_nocache")
        return lg

    def eval_mask(self, skip: np.ndarray, window: Sequence[int], want_logits: bool = False):
        """Parallel candidate evaluation (Section 4.1.2, Eq. 3-4).  window: the tokens at positions
        n - gamma .. n (gamma committed tokens, then the pending token).  Returns (predicted[gamma],
        n_match[, logits[gamma][vocab]]); matchness = n_match / gamma."""
        w = np.ascontiguousarray(window, np.int32)
        gamma = w.size - 1
        skip = np.ascontiguousarray(skip, np.uint8)
        pred = np.empty(max(gamma, 0), np.int32)
        lg = np.empty((gamma, self.vocab), np.float64) if want_logits else None
        nm = C.c_int(0)
        _chk(lib().ora_eval_mask(self._h, _p(skip, C.c_uint8), _p(w, C.c_int32), gamma, _p(pred, C.c_int32),
                                 C.byref(nm), _p(lg, C.c_double) if want_logits else None), "ora_eval_mask")
        return (pred, nm.value, lg) if want_logits else (pred, nm.value)

    TREE_ROWS = 32
    TOPK = 10

    def draft_step_topk(self, skip: np.ndarray, max_k: int, conf_threshold: float, max_width: int = 10):
        """Drafting with the top candidates of every position kept (Section 4.2, strategy 2).
        Returns (levels: list of int32 arrays, level j = candidates of draft position j+1, first =
        the draft token; conf[k])."""
        skip = np.ascontiguousarray(skip, np.uint8)
        cap = max(max_k, 1)
        toks = np.zeros((cap, self.TOPK), np.int32)
        conf = np.zeros(cap, np.float64)
        width = np.zeros(cap, np.int32)
        k = C.c_int(0)
        _chk(lib().ora_draft_step_topk(self._h, _p(skip, C.c_uint8), max_k, conf_threshold, max_width,
                                       _p(toks, C.c_int32), _p(conf, C.c_double),
                                       width.ctypes.data_as(C.POINTER(C.c_int)), C.byref(k)), "ora_draft_step_topk")
        return [toks[j, :width[j]].copy() for j in range(k.value)], conf[:k.value].copy()

    def verify_tree(self, pending: int, levels, want_logits: bool = False):
        """levels: list of candidate arrays (first = spine).  Returns (targets[rows], logits or None)."""
        rows = np.concatenate([[pending]] + [np.asarray(l, np.int32) for l in levels]).astype(np.int32)
        width = np.array([len(l) for l in levels], np.int32)
        tgt = np.empty(rows.size, np.int32)
        lg = np.empty((rows.size, self.vocab), np.float64) if want_logits else None
        _chk(lib().ora_verify_tree(self._h, _p(rows, C.c_int32), width.ctypes.data_as(C.POINTER(C.c_int)), len(levels),
                                   _p(tgt, C.c_int32), _p(lg, C.c_double) if want_logits else None), "ora_verify_tree")
        return tgt, lg

    def rollback(self, new_cache_len: int, pending: int):
        _chk(lib().ora_rollback(self._h, new_cache_len, pending), "ora_rollback")

    # -- speculative sampling
    def prefill_sample(self, prompt: Sequence[int], temperature: float, top_p: float, u: float):
        """Returns (first token, margin)."""
        p = np.ascontiguousarray(prompt, np.int32)
        tok = C.c_int32()
        mg = C.c_double()
        _chk(lib().ora_prefill_sample(self._h, _p(p, C.c_int32), p.size, temperature, top_p, u, C.byref(tok),
                                      C.byref(mg)), "ora_prefill_sample")
        return tok.value, mg.value

    def draft_step_sample(self, skip: np.ndarray, max_k: int, conf_threshold: float, temperature: float, top_p: float,
                          u: Sequence[float]):
        """Returns (draft tokens, conf, margin)."""
        skip = np.ascontiguousarray(skip, np.uint8)
        u = np.ascontiguousarray(u, np.float64)
        assert u.size >= max_k
        cap = max(max_k, 1)
        toks = np.zeros(cap, np.int32)
        conf = np.zeros(cap, np.float64)
        k = C.c_int(0)
        mg = C.c_double()
        _chk(lib().ora_draft_step_sample(self._h, _p(skip, C.c_uint8), max_k, conf_threshold, temperature, top_p,
                                         _p(u, C.c_double), _p(toks, C.c_int32), _p(conf, C.c_double), C.byref(k),
                                         C.byref(mg)), "ora_draft_step_sample")
        return toks[:k.value].copy(), conf[:k.value].copy(), mg.value

    def verify_sample(self, tokens: Sequence[int], temperature: float, top_p: float, u_accept: Sequence[float],
                      u_final: float, want_probs: bool = False):
        """Returns (emitted tokens, probs or None, margin)."""
        t = np.ascontiguousarray(tokens, np.int32)
        k = t.size - 1
        ua = np.ascontiguousarray(u_accept, np.float64)
        assert ua.size >= k
        em = np.zeros(k + 1, np.int32)
        n = C.c_int(0)
        mg = C.c_double()
        pr = np.empty((k + 1, self.vocab), np.float64) if want_probs else None
        _chk(lib().ora_verify_sample(self._h, _p(t, C.c_int32), k, temperature, top_p, _p(ua, C.c_double), u_final,
                                     _p(em, C.c_int32), C.byref(n), _p(pr, C.c_double) if want_probs else None,
                                     C.byref(mg)), "ora_verify_sample")
        return em[:n.value].copy(), pr, mg.value

    def accept_tree(self) -> np.ndarray:
        em = np.empty(self.TREE_ROWS, np.int32)
        n = C.c_int(0)
        _chk(lib().ora_accept_tree(self._h, _p(em, C.c_int32), C.byref(n)), "ora_accept_tree")
        return em[:n.value].copy()

    # -- decoding steps
    def reset(self):
        lib().ora_reset(self._h)

    def prefill(self, prompt: Sequence[int]):
        p = np.ascontiguousarray(prompt, np.int32)
        lg = np.empty(self.vocab, np.float64)
        tok = C.c_int32()
        _chk(lib().ora_prefill(self._h, _p(p, C.c_int32), p.size, C.byref(tok), _p(lg, C.c_double)), "ora_prefill")
        return tok.value, lg

    def draft_step(self, skip: np.ndarray, max_k: int, conf_threshold: float):
        skip = np.ascontiguousarray(skip, np.uint8)
        toks = np.zeros(max(max_k, 1), np.int32)
        conf = np.zeros(max(max_k, 1), np.float64)
        k = C.c_int()
        _chk(lib().ora_draft_step(self._h, _p(skip, C.c_uint8), max_k, conf_threshold, _p(toks, C.c_int32),
                                  _p(conf, C.c_double), C.byref(k)), "ora_draft_step")
        return toks[:k.value].copy(), conf[:k.value].copy()

    def verify(self, tokens: Sequence[int], want_logits: bool = False):
        t = np.ascontiguousarray(tokens, np.int32)
        k = t.size - 1
        tgt = np.zeros(k + 1, np.int32)
        lg = np.empty((k + 1, self.vocab), np.float64) if want_logits else None
        _chk(lib().ora_verify(self._h, _p(t, C.c_int32), k, _p(tgt, C.c_int32),
                              _p(lg, C.c_double) if want_logits else None), "ora_verify")
        return tgt, lg

    def accept(self) -> np.ndarray:
        out = np.zeros(MAX_BLOCK + 1, np.int32)
        n = C.c_int()
        _chk(lib().ora_accept(self._h, _p(out, C.c_int32), C.byref(n)), "ora_accept")
        return out[:n.value].copy()

    @property
    def cache_len(self) -> int:
        return lib().ora_cache_len(self._h)

    @property
    def pending(self) -> int:
        return lib().ora_pending(self._h)

    def stats(self) -> Dict[str, int]:
        a = (C.c_int64 * 4)()
        lib().ora_get_stats(self._h, a)
        return dict(draft_passes=a[0], verify_passes=a[1], accepted=a[2], emitted=a[3])

    def poison_kv(self):
        lib().ora_poison_kv(self._h)

    def read_kv(self, layer: int, pos: int):
        w = self.shape.n_kv_heads * self.shape.head_dim
        k = np.empty(w, np.float32)
        v = np.empty(w, np.float32)
        lib().ora_read_kv(self._h, layer, pos, _p(k, C.c_float), _p(v, C.c_float))
        return k, v


# ---- generation loops -------------------------------------------------------
def generate_ar(o: Oracle, prompt: Sequence[int], n_new: int, want_logits: bool = False):
    """Plain greedy decoding with the target model: the first new token comes
    from the prompt's last row, every further one from a one-row verify."""
    tok, lg = o.prefill(prompt)
    out = [tok]
    logits = [lg]
    while len(out) < n_new:
        tgt, lg = o.verify([o.pending], want_logits)
        o.accept()
        out.append(int(tgt[0]))
        if want_logits:
            logits.append(lg[0])
    return (np.array(out, np.int32), np.stack(logits)) if want_logits else np.array(out, np.int32)


def generate_swift(o: Oracle, prompt: Sequence[int], n_new: int, skip: np.ndarray, max_k: int,
                   conf_threshold: float, poison: bool = False, want_logits: bool = False):
    """Draft-then-verify greedy decoding.  The draft length of a step is capped
    at (tokens still wanted - 1) and by the cache capacity, so exactly n_new
    tokens come out and no draft work is spent past the end.
    Returns (tokens, trace); trace has one dict per decoding step."""
    tok, lg0 = o.prefill(prompt)
    out: List[int] = [tok]
    trace: List[dict] = []
    while len(out) < n_new:
        if poison:
            o.poison_kv()
        k_cap = min(max_k, n_new - len(out) - 1)
        n0 = o.cache_len
        if k_cap > 0:
            d, conf = o.draft_step(skip, k_cap, conf_threshold)
        else:
            d, conf = np.zeros(0, np.int32), np.zeros(0)
        block = np.concatenate([[o.pending], d]).astype(np.int32)
        tgt, lg = o.verify(block, want_logits)
        em = o.accept()
        out.extend(int(t) for t in em)
        trace.append(dict(n=n0, block=block, draft=d, conf=conf, target=tgt, emitted=em, m=len(em) - 1,
                          logits=lg))
    return np.array(out, np.int32), trace


def generate_swift_tree(o: Oracle, prompt: Sequence[int], n_new: int, skip: np.ndarray, max_k: int,
                        conf_threshold: float, max_width: int = 10):
    """Draft-then-verify greedy decoding with dynamic verification (Section 4.2, strategies 1 and 2):
    every draft position is widened to its top candidates and the whole token tree is verified in
    one block.  Returns (tokens, trace)."""
    out = [int(o.prefill(prompt)[0])]
    trace = []
    while len(out) < n_new:
        k_cap = min(max_k, n_new - len(out) - 1)
        n0 = o.cache_len
        levels, conf = o.draft_step_topk(skip, k_cap, conf_threshold, max_width) if k_cap > 0 else ([], np.zeros(0))
        tgt, _ = o.verify_tree(o.pending, levels)
        em = o.accept_tree()
        out.extend(int(t) for t in em)
        trace.append(dict(n=n0, levels=levels, conf=conf, target=tgt, emitted=em, m=len(em) - 1))
    return np.array(out[:n_new], np.int32), trace


def generate_swift_on_the_fly(o: Oracle, opt, prompt: Sequence[int], n_new: int, max_k: int, conf_threshold: float,
                              gamma: int = 32, tree_width: int = 0):
    """Section 4 as a whole for one input: context accumulation with the uniform initial pattern, then
    an optimisation step before every decoding step until the optimiser terminates, then acceleration
    with the retained layer set.  An optimisation step needs gamma committed generated tokens; its
    window is those plus the pending token.  Returns (tokens, trace)."""
    out = [int(o.prefill(prompt)[0])]
    mask = opt.initial_mask()
    done = False
    trace = []
    while len(out) < n_new:
        info = None
        if (not done) and len(out) >= gamma + 1:
            window = np.array(out[len(out) - gamma - 1:], np.int32)
            info = opt.step(o, window)
            mask = info["best"]
            done = info["finished"]
        k_cap = min(max_k, n_new - len(out) - 1)
        n0 = o.cache_len
        if tree_width > 0:
            levels = o.draft_step_topk(mask, k_cap, conf_threshold, tree_width)[0] if k_cap > 0 else []
            o.verify_tree(o.pending, levels)
            em = o.accept_tree()
            n_draft = len(levels)
        else:
            d = o.draft_step(mask, k_cap, conf_threshold)[0] if k_cap > 0 else np.zeros(0, np.int32)
            o.verify(np.concatenate([[o.pending], d]).astype(np.int32))
            em = o.accept()
            n_draft = len(d)
        out.extend(int(t) for t in em)
        trace.append(dict(n=n0, mask=np.array(mask, np.uint8), opt=info, n_draft=n_draft, emitted=em, m=len(em) - 1))
    return np.array(out[:n_new], np.int32), trace


SAMPLE_U_PER_STEP = 31  # uniforms one decoding step may use: 15 draws, 15 acceptance tests, 1 final draw


def generate_swift_sample(o: Oracle, prompt: Sequence[int], n_new: int, skip: np.ndarray, max_k: int,
                          conf_threshold: float, temperature: float, top_p: float, u0: float, U: np.ndarray):
    """Draft-then-verify decoding with speculative sampling.  u0: the uniform of the first token;
    U[s]: the uniforms of decoding step s ([0:15] draft draws, [15:30] acceptance tests, [30] the
    final draw).  Returns (tokens, trace); trace[s]["margin"] says how far the step's decisions
    were from falling differently."""
    tok, mg0 = o.prefill_sample(prompt, temperature, top_p, u0)
    out = [int(tok)]
    trace = []
    s = 0
    while len(out) < n_new:
        k_cap = min(max_k, n_new - len(out) - 1)
        n0 = o.cache_len
        if k_cap > 0:
            d, conf, m1 = o.draft_step_sample(skip, k_cap, conf_threshold, temperature, top_p, U[s, 0:15])
        else:
            d, conf, m1 = np.zeros(0, np.int32), np.zeros(0), 1.0
        block = np.concatenate([[o.pending], d]).astype(np.int32)
        em, _, m2 = o.verify_sample(block, temperature, top_p, U[s, 15:30], float(U[s, 30]))
        out.extend(int(t) for t in em)
        trace.append(dict(n=n0, draft=d, conf=conf, emitted=em, m=len(em) - 1, margin=min(m1, m2),
                          first_margin=mg0))
        s += 1
    return np.array(out[:n_new], np.int32), trace
