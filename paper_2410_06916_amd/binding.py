"""ctypes binding of libswift_hip.so: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

from . import build as _build

F32, BF16 = 0, 1
MAX_BLOCK = 32
MAX_WINDOW = 128   # longest candidate-evaluation window (SWIFT_MAX_WINDOW)
TOPK = 10
KERNEL_CLASSES = {"qkv": 0, "attn": 1, "oproj": 2, "gateup": 3, "down": 4, "lmhead": 5, "other": 6}
_CODES = {-1: "SWIFT_EINVAL", -2: "SWIFT_ECAPACITY", -3: "SWIFT_ESTATE", -4: "SWIFT_EDEVICE"}


class SwiftError(RuntimeError):
    def __init__(self, code: int, what: str, msg: str):
        super().__init__(f"{what}: {_CODES.get(code, code)}: {msg}")
        self.code = code


class ModelConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab",
                                          "max_seq")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("draft_passes", "verify_passes", "accepted", "emitted_by_verify",
                                          "emitted_total")]


_lib = None


class OptConfig(C.Structure):
    _fields_ = [("n_sublayers", C.c_int), ("skip_ratio", C.c_double), ("max_steps", C.c_int), ("max_stale", C.c_int),
                ("stop_matchness", C.c_double), ("seed", C.c_uint64)]


SUGGEST_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.c_int, C.POINTER(C.c_uint8), C.c_double, C.c_int, C.POINTER(C.c_uint8))


def lib():
    """Loads the built library.  There is no fallback: if it is missing it is built with
    hipcc, and if that fails the error propagates."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.lib_path()
    if _build.is_stale():
        # no library yet, or its sources have changed since it was built: never run an old binary
        _build.build()
    # PyTorch ships its own HIP runtime (soname libamdhip64.so.7).  It has to be in the process
    # before this library is loaded so that both resolve to that one runtime; two HIP runtimes in
    # one process do not see each other's device state.
    import torch  # noqa: F401
    L = C.CDLL(path)
    vp, i32p, f32p, u8p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_uint8)
    cfgp = C.POINTER(ModelConfig)
    L.swift_check_config.argtypes = [cfgp]
    L.swift_device_bytes.argtypes = [cfgp, C.POINTER(C.c_uint64)]
    L.swift_expected_speedup.argtypes = [C.c_double] * 3
    L.swift_expected_speedup.restype = C.c_double
    L.swift_match_prefix.argtypes = [i32p, i32p, C.c_int]
    L.swift_pass_bytes.argtypes = [cfgp, u8p, C.c_int, C.c_int, C.POINTER(C.c_uint64)]
    L.swift_last_error.restype = C.c_char_p
    L.swift_create.argtypes = [cfgp, vp, C.c_uint64, vp, C.POINTER(vp)]
    L.swift_destroy.argtypes = [vp]
    L.swift_load_tensor.argtypes = [vp, C.c_char_p, vp, C.c_int, C.c_int64]
    L.swift_prefill.argtypes = [vp, i32p, C.c_int, i32p]
    L.swift_draft_step.argtypes = [vp, u8p, C.c_int, C.c_float, i32p, f32p, C.POINTER(C.c_int)]
    L.swift_verify.argtypes = [vp, i32p, C.c_int, i32p, f32p]
    L.swift_verify_static.argtypes = [vp, i32p, C.c_int, i32p, f32p]
    L.swift_eval_mask.argtypes = [vp, u8p, i32p, C.c_int, i32p, C.POINTER(C.c_int)]
    L.swift_opt_create.argtypes = [C.POINTER(OptConfig), u8p, C.POINTER(vp)]
    L.swift_opt_destroy.argtypes = [vp]
    L.swift_opt_initial_mask.argtypes = [vp, u8p]
    L.swift_opt_candidate.argtypes = [vp, C.c_int, u8p]
    L.swift_opt_set_suggester.argtypes = [vp, SUGGEST_FN, vp, C.c_int]
    L.swift_opt_step.argtypes = [vp, vp, i32p, C.c_int, u8p, C.POINTER(C.c_double), u8p, C.POINTER(C.c_double),
                                 C.POINTER(C.c_int)]
    L.swift_accept.argtypes = [vp, i32p, C.POINTER(C.c_int)]
    L.swift_prefill_sample.argtypes = [vp, i32p, C.c_int, C.c_float, C.c_float, C.c_float, i32p]
    L.swift_draft_step_sample.argtypes = [vp, u8p, C.c_int, C.c_float, C.c_float, C.c_float, f32p, i32p, f32p,
                                          C.POINTER(C.c_int)]
    L.swift_verify_sample.argtypes = [vp, i32p, C.c_int, C.c_float, C.c_float, f32p, C.c_float, i32p,
                                      C.POINTER(C.c_int), f32p]
    L.swift_topk_width.argtypes = [C.c_float]
    L.swift_draft_step_topk.argtypes = [vp, u8p, C.c_int, C.c_float, C.c_int, i32p, f32p, C.POINTER(C.c_int),
                                        C.POINTER(C.c_int)]
    L.swift_verify_tree.argtypes = [vp, i32p, C.POINTER(C.c_int), C.c_int, i32p, f32p]
    L.swift_accept_tree.argtypes = [vp, i32p, C.POINTER(C.c_int)]
    L.swift_rollback.argtypes = [vp, C.c_int, C.c_int32]
    L.swift_get_state.argtypes = [vp, C.POINTER(C.c_int), i32p]
    L.swift_get_stats.argtypes = [vp, C.POINTER(Stats)]
    L.swift_get_config.argtypes = [vp, cfgp]
    L.swift_debug_poison_kv.argtypes = [vp]
    L.swift_debug_read_logits.argtypes = [vp, C.c_int, f32p]
    L.swift_debug_read_kv.argtypes = [vp, C.c_int, C.c_int, f32p, f32p]
    L.swift_debug_tune.argtypes = [vp, C.c_int, C.c_int, C.c_int]
    L.swift_debug_prefill.argtypes = [vp, C.c_int, C.c_int]
    L.swift_debug_attn_path.argtypes = [vp, C.c_int, C.c_int, C.c_char_p, C.c_int]
    L.swift_profile_class.argtypes = [vp, C.c_int]
    L.swift_profile_read.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_double), C.POINTER(C.c_uint64)]
    _lib = L
    return L


def _chk(rc: int, what: str):
    if rc != 0:
        raise SwiftError(rc, what, lib().swift_last_error().decode())


def _p(a: np.ndarray, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def make_config(shape, max_seq: int) -> ModelConfig:
    """shape: any object with n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab,
    rms_eps, rope_theta, dtype ("fp32" | "bf16")."""
    return ModelConfig(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                       shape.vocab, max_seq, shape.rms_eps, shape.rope_theta, F32 if shape.dtype == "fp32" else BF16)


def check_config(cfg: ModelConfig) -> int:
    return lib().swift_check_config(C.byref(cfg))


def device_bytes(cfg: ModelConfig) -> int:
    n = C.c_uint64()
    _chk(lib().swift_device_bytes(C.byref(cfg), C.byref(n)), "swift_device_bytes")
    return n.value


def expected_speedup(M: float, alpha: float, c: float) -> float:
    return lib().swift_expected_speedup(M, alpha, c)


def match_prefix(draft: Sequence[int], target: Sequence[int]) -> int:
    d = np.ascontiguousarray(draft, np.int32)
    t = np.ascontiguousarray(target, np.int32)
    return lib().swift_match_prefix(_p(d, C.c_int32), _p(t, C.c_int32), min(d.size, t.size))


def pass_bytes(cfg: ModelConfig, skip: Optional[np.ndarray], n_ctx: int, rows: int = 1) -> int:
    n = C.c_uint64()
    sp = None
    if skip is not None:
        skip = np.ascontiguousarray(skip, np.uint8)
        if skip.size != 2 * cfg.n_layers:
            raise ValueError(f"skip mask must have {2 * cfg.n_layers} entries")
        sp = _p(skip, C.c_uint8)
    _chk(lib().swift_pass_bytes(C.byref(cfg), sp, n_ctx, rows, C.byref(n)), "swift_pass_bytes")
    return n.value


class SwiftModel:
    """One context: device arena (a torch uint8 tensor), stream (torch's current stream of the
    device at construction) and the C-ABI calls."""

    def __init__(self, shape, max_seq: int, device: str = "cuda:0"):
        import torch
        self.torch = torch
        self.shape = shape
        self.cfg = make_config(shape, max_seq)
        self.device = torch.device(device)
        nbytes = device_bytes(self.cfg)
        torch.cuda.set_device(self.device)
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.arena.data_ptr() + 255) // 256 * 256
        self.stream = torch.cuda.current_stream(self.device)
        self._h = C.c_void_p()
        _chk(lib().swift_create(C.byref(self.cfg), C.c_void_p(base), nbytes, C.c_void_p(self.stream.cuda_stream),
                                C.byref(self._h)), "swift_create")

    def close(self):
        if getattr(self, "_h", None):
            lib().swift_destroy(self._h)
            self._h = C.c_void_p()
            self.arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- weights
    def load_tensor(self, name: str, t):
        torch = self.torch
        t = t.detach().contiguous()
        if t.dtype == torch.float32:
            dt = F32
        elif t.dtype == torch.bfloat16:
            dt = BF16
        else:
            raise TypeError(t.dtype)
        _chk(lib().swift_load_tensor(self._h, name.encode(), C.c_void_p(t.data_ptr()), dt, t.numel()),
             f"swift_load_tensor({name})")

    def load_weights(self, weights):
        for name, t in (weights.items() if hasattr(weights, "items") else weights):
            self.load_tensor(name, t)

    def _mask(self, skip) -> np.ndarray:
        """A skip mask as the library reads it: uint8[2 * n_layers]."""
        skip = np.ascontiguousarray(skip, np.uint8)
        if skip.ndim != 1 or skip.size != 2 * self.cfg.n_layers:
            raise ValueError(f"skip mask must have {2 * self.cfg.n_layers} entries, got {skip.shape}")
        return skip

    # -- decoding path
    def prefill(self, prompt: Sequence[int]) -> int:
        p = np.ascontiguousarray(prompt, np.int32)
        tok = C.c_int32()
        _chk(lib().swift_prefill(self._h, _p(p, C.c_int32), p.size, C.byref(tok)), "swift_prefill")
        return tok.value

    def draft_step(self, skip: np.ndarray, max_k: int, conf_threshold: float):
        skip = self._mask(skip)
        toks = np.zeros(max(max_k, 1), np.int32)
        conf = np.zeros(max(max_k, 1), np.float32)
        k = C.c_int()
        _chk(lib().swift_draft_step(self._h, _p(skip, C.c_uint8), max_k, conf_threshold, _p(toks, C.c_int32),
                                    _p(conf, C.c_float), C.byref(k)), "swift_draft_step")
        return toks[:k.value].copy(), conf[:k.value].copy()

    def verify(self, tokens: Sequence[int], want_logits: bool = False):
        t = np.ascontiguousarray(tokens, np.int32)
        k = t.size - 1
        tgt = np.zeros(k + 1, np.int32)
        lg = np.empty((k + 1, self.cfg.vocab), np.float32) if want_logits else None
        _chk(lib().swift_verify(self._h, _p(t, C.c_int32), k, _p(tgt, C.c_int32),
                                _p(lg, C.c_float) if want_logits else None), "swift_verify")
        return tgt, lg

    def verify_static(self, tokens: Sequence[int], want_logits: bool = False):
        """swift_verify_static: verification whose kernels' scratch lies in the library's static device array."""
        t = np.ascontiguousarray(tokens, np.int32)
        k = t.size - 1
        tgt = np.zeros(k + 1, np.int32)
        lg = np.empty((k + 1, self.cfg.vocab), np.float32) if want_logits else None
        _chk(lib().swift_verify_static(self._h, _p(t, C.c_int32), k, _p(tgt, C.c_int32),
                                       _p(lg, C.c_float) if want_logits else None), "swift_verify_static")
        return tgt, lg

    def accept(self) -> np.ndarray:
        out = np.zeros(MAX_BLOCK, np.int32)
        n = C.c_int()
        _chk(lib().swift_accept(self._h, _p(out, C.c_int32), C.byref(n)), "swift_accept")
        return out[:n.value].copy()

    def draft_step_topk(self, skip: np.ndarray, max_k: int, conf_threshold: float, max_width: int = 10):
        """Drafting that keeps the top candidates of every position (Section 4.2, second strategy).
        Returns (levels: one int32 array of candidates per draft position, first = the draft token; conf[k])."""
        skip = self._mask(skip)
        cap = max(max_k, 1)
        toks = np.zeros((cap, TOPK), np.int32)
        conf = np.zeros(cap, np.float32)
        width = np.zeros(cap, np.intc)
        k = C.c_int()
        _chk(lib().swift_draft_step_topk(self._h, _p(skip, C.c_uint8), max_k, conf_threshold, max_width,
                                         _p(toks, C.c_int32), _p(conf, C.c_float), _p(width, C.c_int), C.byref(k)),
             "swift_draft_step_topk")
        return [toks[j, :width[j]].copy() for j in range(k.value)], conf[:k.value].copy()

    def verify_tree(self, levels, want_logits: bool = False):
        """levels: candidate arrays per draft position (first = the draft token).  The block is the pending
        token followed by the levels.  Returns (targets[rows], logits or None)."""
        rows = np.concatenate([[self.pending]] + [np.asarray(l, np.int32) for l in levels]).astype(np.int32)
        width = np.array([len(l) for l in levels], np.intc)
        tgt = np.zeros(rows.size, np.int32)
        lg = np.empty((rows.size, self.cfg.vocab), np.float32) if want_logits else None
        _chk(lib().swift_verify_tree(self._h, _p(rows, C.c_int32), _p(width, C.c_int) if len(levels) else None,
                                     len(levels), _p(tgt, C.c_int32), _p(lg, C.c_float) if want_logits else None),
             "swift_verify_tree")
        return tgt, lg

    def accept_tree(self) -> np.ndarray:
        out = np.zeros(MAX_BLOCK, np.int32)
        n = C.c_int()
        _chk(lib().swift_accept_tree(self._h, _p(out, C.c_int32), C.byref(n)), "swift_accept_tree")
        return out[:n.value].copy()

    def prefill_sample(self, prompt: Sequence[int], temperature: float, top_p: float, u: float) -> int:
        p = np.ascontiguousarray(prompt, np.int32)
        tok = C.c_int32()
        _chk(lib().swift_prefill_sample(self._h, _p(p, C.c_int32), p.size, temperature, top_p, u, C.byref(tok)),
             "swift_prefill_sample")
        return tok.value

    def draft_step_sample(self, skip: np.ndarray, max_k: int, conf_threshold: float, temperature: float, top_p: float,
                          u: Sequence[float]):
        """Sampled drafting (speculative sampling): u = the uniforms of the draws.  Returns (tokens, conf)."""
        skip = self._mask(skip)
        u = np.ascontiguousarray(u, np.float32)
        assert u.size >= max_k
        toks = np.zeros(max(max_k, 1), np.int32)
        conf = np.zeros(max(max_k, 1), np.float32)
        k = C.c_int()
        _chk(lib().swift_draft_step_sample(self._h, _p(skip, C.c_uint8), max_k, conf_threshold, temperature, top_p,
                                           _p(u, C.c_float), _p(toks, C.c_int32), _p(conf, C.c_float), C.byref(k)),
             "swift_draft_step_sample")
        return toks[:k.value].copy(), conf[:k.value].copy()

    def verify_sample(self, tokens: Sequence[int], temperature: float, top_p: float, u_accept: Sequence[float],
                      u_final: float, want_probs: bool = False):
        """Verification + acceptance by speculative sampling.  Returns (emitted, probs or None)."""
        t = np.ascontiguousarray(tokens, np.int32)
        k = t.size - 1
        ua = np.ascontiguousarray(u_accept, np.float32)
        assert ua.size >= k
        em = np.zeros(k + 1, np.int32)
        n = C.c_int()
        pr = np.empty((k + 1, self.cfg.vocab), np.float32) if want_probs else None
        _chk(lib().swift_verify_sample(self._h, _p(t, C.c_int32), k, temperature, top_p,
                                       _p(ua, C.c_float) if k else None, u_final, _p(em, C.c_int32), C.byref(n),
                                       _p(pr, C.c_float) if want_probs else None), "swift_verify_sample")
        return em[:n.value].copy(), pr

    def eval_mask(self, skip: np.ndarray, window: Sequence[int]):
        """Candidate evaluation (Section 4.1.2): window = last gamma committed tokens + the pending
        token.  Returns (predicted[gamma], n_match)."""
        w = np.ascontiguousarray(window, np.int32)
        gamma = w.size - 1
        skip = self._mask(skip)
        pred = np.empty(max(gamma, 0), np.int32)
        nm = C.c_int(0)
        _chk(lib().swift_eval_mask(self._h, _p(skip, C.c_uint8), _p(w, C.c_int32), gamma, _p(pred, C.c_int32),
                                   C.byref(nm)), "swift_eval_mask")
        return pred, nm.value

    def rollback(self, new_cache_len: int, pending: int):
        _chk(lib().swift_rollback(self._h, new_cache_len, pending), "swift_rollback")

    @property
    def cache_len(self) -> int:
        n = C.c_int()
        _chk(lib().swift_get_state(self._h, C.byref(n), None), "swift_get_state")
        return n.value

    @property
    def pending(self) -> int:
        t = C.c_int32()
        _chk(lib().swift_get_state(self._h, None, C.byref(t)), "swift_get_state")
        return t.value

    def stats(self) -> Dict[str, int]:
        s = Stats()
        _chk(lib().swift_get_stats(self._h, C.byref(s)), "swift_get_stats")
        return {n: getattr(s, n) for n, _ in Stats._fields_}

    # -- hooks
    def poison_kv(self):
        _chk(lib().swift_debug_poison_kv(self._h), "swift_debug_poison_kv")

    def read_logits(self, row: int = 0) -> np.ndarray:
        out = np.empty(self.cfg.vocab, np.float32)
        _chk(lib().swift_debug_read_logits(self._h, row, _p(out, C.c_float)), "swift_debug_read_logits")
        return out

    def read_kv(self, layer: int, pos: int):
        w = self.cfg.n_kv_heads * self.cfg.head_dim
        k = np.empty(w, np.float32)
        v = np.empty(w, np.float32)
        _chk(lib().swift_debug_read_kv(self._h, layer, pos, _p(k, C.c_float), _p(v, C.c_float)), "swift_debug_read_kv")
        return k, v

    def attn_path(self, rows: int, tree: bool = False) -> str:
        """Name of the attention kernel instance a block of `rows` rows takes in this context."""
        buf = C.create_string_buffer(96)
        _chk(lib().swift_debug_attn_path(self._h, rows, 1 if tree else 0, buf, 96), "swift_debug_attn_path")
        return buf.value.decode()

    def tune(self, name: str, waves_per_row_group: int = 0, workgroups: int = 0):
        _chk(lib().swift_debug_tune(self._h, KERNEL_CLASSES[name], waves_per_row_group, workgroups), "swift_debug_tune")

    def prefill_blocks(self, sub_blocks: int = 0, tiling: int = 0):
        """How prefill walks a prompt (bf16 models): 0 = default macro blocks, 1..8 = at most that many 64-row
        sub-blocks per sweep over the weights, -1 = one 64-row block per sweep; tiling: 0 = automatic, 1..6 = the
        workgroup tile of the blocked matrix product (see swift_debug_prefill)."""
        _chk(lib().swift_debug_prefill(self._h, sub_blocks, tiling), "swift_debug_prefill")

    def profile_class(self, name: Optional[str]):
        _chk(lib().swift_profile_class(self._h, -1 if name is None else KERNEL_CLASSES[name]), "swift_profile_class")

    def profile_read(self):
        n, ms, b = C.c_int64(), C.c_double(), C.c_uint64()
        _chk(lib().swift_profile_read(self._h, C.byref(n), C.byref(ms), C.byref(b)), "swift_profile_read")
        return n.value, ms.value, b.value


class Optimizer:
    """Optimisation phase on top of SwiftModel.eval_mask (argument marshalling only): uniform initial
    pattern, random-search candidates, best candidate retained, termination rules."""

    def __init__(self, n_sublayers: int, skip_ratio: float, max_steps: int = 1000, max_stale: int = 300,
                 stop_matchness: float = 0.95, seed: int = 0, eligible: Optional[np.ndarray] = None):
        self.n = n_sublayers
        cfg = OptConfig(n_sublayers, skip_ratio, max_steps, max_stale, stop_matchness, seed)
        el = None if eligible is None else np.ascontiguousarray(eligible, np.uint8)
        h = C.c_void_p()
        _chk(lib().swift_opt_create(C.byref(cfg), None if el is None else _p(el, C.c_uint8), C.byref(h)), "swift_opt_create")
        self._h = h
        self._cb = None

    def close(self):
        if self._h:
            lib().swift_opt_destroy(self._h)
            self._h = None

    def initial_mask(self) -> np.ndarray:
        m = np.zeros(self.n, np.uint8)
        _chk(lib().swift_opt_initial_mask(self._h, _p(m, C.c_uint8)), "swift_opt_initial_mask")
        return m

    def candidate(self, step: int) -> np.ndarray:
        m = np.zeros(self.n, np.uint8)
        _chk(lib().swift_opt_candidate(self._h, step, _p(m, C.c_uint8)), "swift_opt_candidate")
        return m

    def set_suggester(self, fn, interval: int):
        """fn(step, best_mask, best_matchness) -> candidate mask or None (None: random search)."""
        def tramp(_user, step, best, best_score, n, out):
            r = fn(step, np.ctypeslib.as_array(best, (n,)).copy(), best_score)
            if r is None:
                return 1
            out_arr = np.ctypeslib.as_array(out, (n,))
            out_arr[:] = np.asarray(r, np.uint8)
            return 0
        self._cb = SUGGEST_FN(tramp) if fn else SUGGEST_FN(0)
        _chk(lib().swift_opt_set_suggester(self._h, self._cb if fn else C.cast(None, SUGGEST_FN), None, interval),
             "swift_opt_set_suggester")

    def step(self, model: "SwiftModel", window: Sequence[int]):
        w = np.ascontiguousarray(window, np.int32)
        cand = np.zeros(self.n, np.uint8)
        best = np.zeros(self.n, np.uint8)
        cs, bs, fin = C.c_double(), C.c_double(), C.c_int()
        _chk(lib().swift_opt_step(model._h, self._h, _p(w, C.c_int32), w.size - 1, _p(cand, C.c_uint8), C.byref(cs),
                                  _p(best, C.c_uint8), C.byref(bs), C.byref(fin)), "swift_opt_step")
        return dict(candidate=cand, score=cs.value, best=best, best_score=bs.value, finished=bool(fin.value))
