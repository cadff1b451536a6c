"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and its host-side logic (configuration checks, arena sizing, byte
accounting, prefix matching, Eq. 6, argument validation) behaves as documented.
No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import synthetic_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def P():
    import paper_2410_06916_amd as P
    P.lib()
    return P


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "swift.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(swift_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(P):
    names = _declared_symbols()
    assert len(names) >= 18
    L = P.lib()
    for n in names:
        assert hasattr(L, n), n


def test_config_checks(P):
    from paper_2410_06916_amd import binding as B
    for w in si.WORKLOADS.values():
        assert P.check_config(B.make_config(w.shape, w.n_prompt + w.n_new + 16)) == 0
    bad = B.make_config(si.TINY, 128)
    bad.head_dim = 48
    assert P.check_config(bad) == -1
    bad = B.make_config(si.TINY, 128)
    bad.n_kv_heads = 3
    assert P.check_config(bad) == -1
    bad = B.make_config(si.TINY, 0)
    assert P.check_config(bad) == -1
    bad = B.make_config(si.TINY, 128)
    bad.dtype = 7
    assert P.check_config(bad) == -1
    assert P.lib().swift_check_config(None) == -1
    with pytest.raises(P.SwiftError):
        P.device_bytes(bad)


def test_arena_size_covers_weights_and_cache(P):
    from paper_2410_06916_amd import binding as B
    s = si.LLAMA2_7B
    max_seq = 1024
    n = P.device_bytes(B.make_config(s, max_seq))
    weights = 2 * (2 * s.vocab * s.hidden + s.n_layers * (s.attn_sublayer_elems() + s.mlp_sublayer_elems()))
    kv = 2 * s.n_layers * 2 * s.kv_dim * max_seq
    assert weights + kv < n < weights + kv + 500e6   # + staging for the largest tensor, activations, tables


def test_pass_bytes_accounting(P):
    from paper_2410_06916_amd import binding as B
    s = si.LLAMA2_7B
    cfg = B.make_config(s, 1024)
    full = P.pass_bytes(cfg, None, 0, 1)
    assert abs(full - 13.21e9) < 0.02e9          # stack + LM head of the 7B shape in bf16
    none = P.pass_bytes(cfg, np.zeros(64, np.uint8), 0, 1)
    assert none == full
    m = np.zeros(64, np.uint8)
    m[2 * 5] = 1
    assert full - P.pass_bytes(cfg, m, 0, 1) == 2 * s.attn_sublayer_elems() + 4 * s.hidden + 2 * 2 * s.kv_dim
    m = np.zeros(64, np.uint8)
    m[2 * 5 + 1] = 1
    assert full - P.pass_bytes(cfg, m, 0, 1) == 2 * s.mlp_sublayer_elems() + 4 * s.hidden
    # key/value traffic: 512 KB per cached token over the 32 layers
    assert P.pass_bytes(cfg, None, 100, 1) - full == 100 * 2 * 2 * s.kv_dim * s.n_layers
    everything = np.ones(64, np.uint8)
    assert P.pass_bytes(cfg, everything, 500, 1) == 2 * s.vocab * s.hidden + 4 * s.hidden + 2 * s.hidden


def test_match_prefix_and_eq6(P, oracle_lib):
    rng = np.random.default_rng(0)
    for _ in range(200):
        k = int(rng.integers(0, 12))
        d = rng.integers(0, 3, k)
        t = rng.integers(0, 3, k)
        want = 0
        while want < k and d[want] == t[want]:
            want += 1
        assert P.match_prefix(d, t) == want
    assert P.lib().swift_match_prefix(None, None, 3) == 0
    # the paper's Table 4 values (fixture shared with the oracle pin)
    from tests.test_oracle_pins import _table4
    for _, _, r, M, alpha, printed in _table4():
        assert abs(P.expected_speedup(M, alpha, 1 - r) - printed) <= 0.005 + 1e-9


def test_null_and_range_arguments_are_rejected_without_a_device(P):
    L = P.lib()
    vp = C.c_void_p
    assert L.swift_destroy(None) == -1
    assert L.swift_prefill(None, None, 0, None) == -1
    assert L.swift_draft_step(None, None, 1, 0.5, None, None, None) == -1
    assert L.swift_verify(None, None, 0, None, None) == -1
    assert L.swift_accept(None, None, None) == -1
    assert L.swift_rollback(None, 0, 0) == -1
    assert L.swift_get_stats(None, None) == -1
    assert L.swift_load_tensor(None, b"embed", None, 0, 0) == -1
    assert L.swift_debug_prefill(None, 0, 0) == -1
    out = vp()
    from paper_2410_06916_amd import binding as B
    cfg = B.make_config(si.TINY, 64)
    assert L.swift_create(C.byref(cfg), None, 0, None, C.byref(out)) == -1      # null arena
    assert L.swift_create(C.byref(cfg), vp(4096 + 8), 1 << 40, None, C.byref(out)) == -1   # misaligned arena
    assert L.swift_create(C.byref(cfg), vp(4096), 16, None, C.byref(out)) == -2  # arena too small
    assert b"arena" in L.swift_last_error()


def test_new_entry_points_reject_null_contexts_without_a_device(P):
    """Dynamic verification, speculative sampling, candidate evaluation: argument checks come first."""
    L = P.lib()
    assert L.swift_eval_mask(None, None, None, 4, None, None) == -1
    assert L.swift_draft_step_topk(None, None, 1, 0.5, 10, None, None, None, None) == -1
    assert L.swift_verify_tree(None, None, None, 0, None, None) == -1
    assert L.swift_accept_tree(None, None, None) == -1
    assert L.swift_prefill_sample(None, None, 0, 0.6, 0.95, 0.5, None) == -1
    assert L.swift_draft_step_sample(None, None, 1, 0.5, 0.6, 0.95, None, None, None, None) == -1
    assert L.swift_verify_sample(None, None, 0, 0.6, 0.95, None, 0.5, None, None, None) == -1
    # the band table of dynamic verification (Section 4.2) is host arithmetic
    assert [L.swift_topk_width(p) for p in (0.01, 0.5, 0.51, 0.8, 0.81, 0.95, 0.96, 1.0)] == [10, 10, 5, 5, 3, 3, 1, 1]


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)
