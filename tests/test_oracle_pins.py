"""Pins of the CPU oracle's building blocks against things that are not the
oracle: values the paper prints, closed forms, textbook special cases and a
library-routine (numpy matmul) rewrite of degenerate cases.  CPU only."""
import math
import os

import numpy as np
import pytest
import torch

import synthetic_inputs as si
from tests import helpers as hp

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- Eq. 6
def _table4():
    rows = []
    with open(os.path.join(GOLDEN, "table4_expected_speedup.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            p = line.split()
            rows.append((p[0], p[1], float(p[2]), float(p[3]), float(p[4]), float(p[5])))
    return rows


def test_eq6_reproduces_table4(oracle_lib):
    rows = _table4()
    assert len(rows) == 9
    for model, task, r, M, alpha, printed in rows:
        got = oracle_lib.expected_speedup(M, alpha, 1.0 - r)
        assert abs(got - printed) <= 0.005 + 1e-9, (model, task, got, printed)


def test_eq6_limits(oracle_lib):
    # vanilla decoding: one token per target pass -> no speedup whatever alpha, c
    assert oracle_lib.expected_speedup(1.0, 0.3, 0.7) == pytest.approx(1.0)
    # free, perfect drafts: speedup = tokens per target pass
    assert oracle_lib.expected_speedup(5.0, 1.0, 0.0) == pytest.approx(5.0)
    # both printed forms of Eq. 6 agree
    M, a, c = 4.34, 0.99, 0.55
    assert oracle_lib.expected_speedup(M, a, c) == pytest.approx(M / ((M - 1) * c / a + 1), rel=1e-12)


# ---------------------------------------------------------------- arg-max / confidence
def test_confidence_uniform_and_dominant(oracle_lib):
    tok, p = oracle_lib.argmax_conf(np.full(1000, 3.25))
    assert tok == 0 and p == pytest.approx(1.0 / 1000, rel=1e-12)
    lg = np.zeros(50)
    lg[17] = 80.0
    tok, p = oracle_lib.argmax_conf(lg)
    assert tok == 17 and p == pytest.approx(1.0, abs=1e-12)
    # two equal maxima: lowest index wins, probability 1/2 each (others negligible)
    lg = np.full(10, -100.0)
    lg[3] = lg[7] = 2.0
    tok, p = oracle_lib.argmax_conf(lg)
    assert tok == 3 and p == pytest.approx(0.5, rel=1e-9)
    # softmax against scipy's log-sum-exp
    from scipy.special import logsumexp
    rng = np.random.default_rng(0)
    lg = (rng.normal(size=300) * 3).astype(np.float32).astype(np.float64)
    tok, p = oracle_lib.argmax_conf(lg)
    assert tok == int(np.argmax(lg)) and p == pytest.approx(math.exp(lg.max() - logsumexp(lg)), rel=1e-12)


def test_argmax_decided_in_fp32(oracle_lib):
    # 1 + 1e-9 and 1 are the same fp32 number: a tie, so the lower index wins
    lg = np.array([0.0, 1.0, 1.0 + 1e-9, 0.5])
    assert oracle_lib.argmax_conf(lg)[0] == 1
    lg = np.array([0.0, 1.0, 1.0 + 1e-6, 0.5])
    assert oracle_lib.argmax_conf(lg)[0] == 2


def test_argmax_of_a_row_without_a_maximum_is_token_zero(oracle_lib):
    """A row of NaN or of -inf only has no element that compares greater than another: the scan that starts at
    index 0 and moves on strict improvement stays at 0 (the rule the library's kernel follows too, so that
    no out-of-range id is ever fed back as an embedding index)."""
    assert oracle_lib.argmax_conf(np.full(40, np.nan))[0] == 0
    assert oracle_lib.argmax_conf(np.full(40, -np.inf))[0] == 0
    lg = np.full(40, np.nan)
    lg[0] = -np.inf
    lg[5] = -3.0            # the first element that compares greater than index 0's wins
    assert oracle_lib.argmax_conf(lg)[0] == 5


# ---------------------------------------------------------------- RMSNorm
def test_rmsnorm_properties(oracle_lib):
    rng = np.random.default_rng(1)
    x = rng.normal(size=64)
    g = np.ones(64)
    y = oracle_lib.rmsnorm(x, g, 0.0)
    assert np.sqrt(np.mean(y * y)) == pytest.approx(1.0, rel=1e-12)          # unit RMS
    assert np.allclose(oracle_lib.rmsnorm(7.5 * x, g, 0.0), y, rtol=1e-12)   # scale invariance
    g2 = g.copy()
    g2[5] = 2.0
    y2 = oracle_lib.rmsnorm(x, g2, 0.0)
    assert y2[5] == pytest.approx(2 * y[5]) and np.allclose(np.delete(y2, 5), np.delete(y, 5))
    # constant vector: a / sqrt(a^2 + eps), eps inside the root and added to the MEAN square
    a, eps = 0.01, 1e-3
    assert np.allclose(oracle_lib.rmsnorm(np.full(8, a), np.ones(8), eps), a / math.sqrt(a * a + eps), rtol=1e-12)
    assert np.all(oracle_lib.rmsnorm(np.zeros(8), np.ones(8), 1e-6) == 0.0)


# ---------------------------------------------------------------- RoPE
def test_rope_worked_example(oracle_lib):
    c1, s1 = float(np.float32(math.cos(1.0))), float(np.float32(math.sin(1.0)))
    # d = 4: pairs (0,2) and (1,3); frequencies 1 and theta^(-1/2) = 0.01
    assert np.allclose(oracle_lib.rope([1, 0, 0, 0], 1, 1e4), [c1, 0, s1, 0], atol=1e-15)
    assert np.allclose(oracle_lib.rope([0, 0, 1, 0], 1, 1e4), [-s1, 0, c1, 0], atol=1e-15)
    assert np.allclose(oracle_lib.rope([0, 1, 0, 0], 100, 1e4), [0, c1, 0, s1], atol=1e-7)
    assert np.allclose(oracle_lib.rope([0, 0, 0, 1], 100, 1e4), [0, -s1, 0, c1], atol=1e-7)


def test_rope_properties(oracle_lib):
    rng = np.random.default_rng(2)
    q, k = rng.normal(size=32), rng.normal(size=32)
    assert np.array_equal(oracle_lib.rope(q, 0, 1e4), q)                          # position 0 = identity
    assert np.linalg.norm(oracle_lib.rope(q, 37, 1e4)) == pytest.approx(np.linalg.norm(q), rel=1e-6)
    d1 = oracle_lib.rope(q, 9, 1e4) @ oracle_lib.rope(k, 4, 1e4)
    d2 = oracle_lib.rope(q, 25, 1e4) @ oracle_lib.rope(k, 20, 1e4)
    d3 = oracle_lib.rope(q, 5, 1e4) @ k
    assert d1 == pytest.approx(d2, abs=1e-5) and d1 == pytest.approx(d3, abs=1e-5)  # depends on p - u only
    assert abs(d1 - q @ k) > 1e-3                                                    # and does depend on it


# ---------------------------------------------------------------- attention
def test_attend_special_cases(oracle_lib):
    rng = np.random.default_rng(3)
    d = 8
    q = rng.normal(size=d)
    v = rng.normal(size=(5, d)).astype(np.float32)
    k = rng.normal(size=(5, d)).astype(np.float32)
    assert np.allclose(oracle_lib.attend(q, k[:1], v[:1]), v[0])                   # one slot -> its value
    ksame = np.repeat(k[:1], 5, axis=0)
    assert np.allclose(oracle_lib.attend(q, ksame, v), v.astype(np.float64).mean(axis=0), rtol=1e-12)  # equal keys -> mean
    # 1/sqrt(d) scaling: d = 4, q.k = (2, 0) -> scores (1, 0) -> weights e/(1+e), 1/(1+e)
    q4 = np.array([2.0, 0, 0, 0])
    k4 = np.array([[1, 0, 0, 0], [0, 0, 0, 0]], np.float32)
    v4 = np.array([[1, 0, 0, 0], [0, 1, 0, 0]], np.float32)
    e = math.e
    assert np.allclose(oracle_lib.attend(q4, k4, v4), [e / (1 + e), 1 / (1 + e), 0, 0], rtol=1e-12)
    # general case against scipy softmax + matmul
    from scipy.special import softmax
    want = softmax(k.astype(np.float64) @ q / math.sqrt(d)) @ v.astype(np.float64)
    assert np.allclose(oracle_lib.attend(q, k, v), want, rtol=1e-12)


def test_swiglu(oracle_lib):
    assert oracle_lib.swiglu(0.0, 5.0) == 0.0
    assert oracle_lib.swiglu(1.0, 1.0) == pytest.approx(0.7310585786300049, rel=1e-12)
    assert oracle_lib.swiglu(1.0, 2.0) == pytest.approx(2 * 0.7310585786300049, rel=1e-12)   # first arg is gated
    assert oracle_lib.swiglu(2.0, 1.0) == pytest.approx(2 / (1 + math.exp(-2)), rel=1e-12)
    assert oracle_lib.swiglu(40.0, 3.0) == pytest.approx(120.0, rel=1e-12)
    assert oracle_lib.swiglu(-40.0, 3.0) == pytest.approx(0.0, abs=1e-12)


def test_match_prefix(oracle_lib):
    assert oracle_lib.match_prefix([5, 6, 7], [5, 6, 7]) == 3
    assert oracle_lib.match_prefix([5, 6, 7], [5, 9, 7]) == 1     # a later coincidence does not count
    assert oracle_lib.match_prefix([5, 6, 7], [4, 6, 7]) == 0
    assert oracle_lib.match_prefix([], []) == 0


# ---------------------------------------------------------------- model-level closed forms
def _np(w):
    return {k: v.float().numpy().astype(np.float64) for k, v in w.items()}


def _rms(x, g, eps):
    return x / np.sqrt(np.mean(x * x) + eps) * g


def test_single_token_one_layer_closed_form(oracle_lib):
    """One token at position 0: the rotation is the identity and the softmax over
    one slot is 1, so the layer collapses to matrix products (numpy matmul)."""
    s = hp.ONE_LAYER
    w = hp.shaped_weights(s, seed=5, branch_scale=1.0, head_scale=1.0)
    o = oracle_lib.Oracle(s, 8)
    o.set_weights(w)
    n = _np(w)
    tok = 11
    x = n["embed"][tok]
    xh = _rms(x, n["l0.attn_norm"], s.rms_eps)
    v = (n["l0.wv"] @ xh).astype(np.float32).astype(np.float64)          # value cache is fp32 here
    group = s.n_q_heads // s.n_kv_heads
    att = np.concatenate([v[(h // group) * s.head_dim:(h // group + 1) * s.head_dim] for h in range(s.n_q_heads)])
    x = x + n["l0.wo"] @ att
    xh = _rms(x, n["l0.mlp_norm"], s.rms_eps)
    g, u = n["l0.wg"] @ xh, n["l0.wu"] @ xh
    x = x + n["l0.wd"] @ (g / (1 + np.exp(-g)) * u)
    want = n["lm_head"] @ _rms(x, n["final_norm"], s.rms_eps)
    got = o.forward_row(tok, 0)
    assert np.allclose(got, want, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("skip_attn,skip_mlp", [(1, 0), (0, 1)])
def test_single_sublayer_masks_delete_exactly_that_sublayer(oracle_lib, skip_attn, skip_mlp):
    """Mask entry 2l bypasses the attention sublayer of layer l and entry 2l+1 its
    MLP (Section 3.1 counts both kinds in z): the same collapse as above with the
    corresponding residual branch removed."""
    s = hp.ONE_LAYER
    w = hp.shaped_weights(s, seed=5, branch_scale=1.0, head_scale=1.0)
    o = oracle_lib.Oracle(s, 8)
    o.set_weights(w)
    n = _np(w)
    tok = 23
    x = n["embed"][tok]
    if not skip_attn:
        xh = _rms(x, n["l0.attn_norm"], s.rms_eps)
        v = (n["l0.wv"] @ xh).astype(np.float32).astype(np.float64)
        group = s.n_q_heads // s.n_kv_heads
        att = np.concatenate([v[(h // group) * s.head_dim:(h // group + 1) * s.head_dim]
                              for h in range(s.n_q_heads)])
        x = x + n["l0.wo"] @ att
    if not skip_mlp:
        xh = _rms(x, n["l0.mlp_norm"], s.rms_eps)
        g, u = n["l0.wg"] @ xh, n["l0.wu"] @ xh
        x = x + n["l0.wd"] @ (g / (1 + np.exp(-g)) * u)
    want = n["lm_head"] @ _rms(x, n["final_norm"], s.rms_eps)
    got = o.forward_row(tok, 0, np.array([skip_attn, skip_mlp], np.uint8))
    assert np.allclose(got, want, rtol=1e-10, atol=1e-12)
    full = o.forward_row(tok, 0)
    assert not np.allclose(got, full, rtol=1e-6)


def test_all_skipped_draft_is_head_of_embedding(oracle_lib):
    """With every sublayer skipped the draft logits are W_lm . rmsnorm(E[prev]),
    whatever the position and the cache contents."""
    s = hp.SMALL_GQA
    w = hp.shaped_weights(s, seed=6)
    o = oracle_lib.Oracle(s, 32)
    o.set_weights(w)
    n = _np(w)
    skip = np.ones(2 * s.n_layers, np.uint8)
    for tok, pos in ((3, 0), (150, 17)):
        want = n["lm_head"] @ _rms(n["embed"][tok], n["final_norm"], s.rms_eps)
        assert np.allclose(o.forward_row(tok, pos, skip), want, rtol=1e-12)


def _numpy_forward(shape, n, tokens, kv_round):
    """Vectorised float64 forward of a whole sequence with library matmuls
    (second implementation of the published LLaMA block, used on tiny inputs)."""
    H, d, nq, nkv = shape.hidden, shape.head_dim, shape.n_q_heads, shape.n_kv_heads
    T = len(tokens)
    X = n["embed"][tokens]
    pos = np.arange(T)[:, None]
    freq = shape.rope_theta ** (-2.0 * np.arange(d // 2) / d)
    cos = np.cos(pos * freq).astype(np.float32).astype(np.float64)
    sin = np.sin(pos * freq).astype(np.float32).astype(np.float64)

    def rot(M, heads):
        M = M.reshape(T, heads, d)
        a, b = M[..., :d // 2], M[..., d // 2:]
        return np.concatenate([a * cos[:, None] - b * sin[:, None], b * cos[:, None] + a * sin[:, None]], -1)

    def norm(X, g):
        return X / np.sqrt(np.mean(X * X, -1, keepdims=True) + shape.rms_eps) * g

    for l in range(shape.n_layers):
        Xh = norm(X, n[f"l{l}.attn_norm"])
        Q = rot(Xh @ n[f"l{l}.wq"].T, nq)
        K = kv_round(rot(Xh @ n[f"l{l}.wk"].T, nkv))
        V = kv_round((Xh @ n[f"l{l}.wv"].T).reshape(T, nkv, d))
        K = np.repeat(K, nq // nkv, axis=1)
        V = np.repeat(V, nq // nkv, axis=1)
        S = np.einsum("thd,uhd->htu", Q, K) / math.sqrt(d)
        S = np.where(np.tril(np.ones((T, T), bool)), S, -np.inf)
        A = np.exp(S - S.max(-1, keepdims=True))
        A /= A.sum(-1, keepdims=True)
        O = np.einsum("htu,uhd->thd", A, V).reshape(T, nq * d)
        X = X + O @ n[f"l{l}.wo"].T
        Xh = norm(X, n[f"l{l}.mlp_norm"])
        G, U = Xh @ n[f"l{l}.wg"].T, Xh @ n[f"l{l}.wu"].T
        X = X + (G / (1 + np.exp(-G)) * U) @ n[f"l{l}.wd"].T
    return norm(X, n["final_norm"]) @ n["lm_head"].T


@pytest.mark.parametrize("shape", [hp.SMALL_GQA, hp.SMALL_GQA_BF16], ids=lambda s: s.name)
def test_cached_forward_matches_numpy_sequence_forward(oracle_lib, shape):
    w = hp.shaped_weights(shape, seed=7, branch_scale=1.0, head_scale=1.0)
    o = oracle_lib.Oracle(shape, 16)
    o.set_weights(w)
    tokens = si.uniform_ids(3, 9, shape.vocab)
    if shape.dtype == "fp32":
        kv_round = lambda a: a.astype(np.float32).astype(np.float64)
    else:
        kv_round = lambda a: torch.from_numpy(a.astype(np.float32)).bfloat16().float().numpy().astype(np.float64)
    want = _numpy_forward(shape, _np(w), tokens, kv_round)
    for t, tok in enumerate(tokens):
        got = o.forward_row(int(tok), t)
        # fp32 cache: only summation order differs.  bf16 cache: a key/value within an ulp of
        # a rounding boundary may round the other way in the other summation order.
        tol = 1e-9 if shape.dtype == "fp32" else 2e-3
        assert np.max(np.abs(got - want[t])) <= tol * np.max(np.abs(want[t])), t


def test_bf16_cache_holds_bf16_values(oracle_lib):
    shape = hp.SMALL_GQA_BF16
    o = oracle_lib.Oracle(shape, 8)
    o.set_weights(hp.shaped_weights(shape, seed=8))
    o.forward_row(5, 0)
    o.forward_row(9, 1)
    for l in range(shape.n_layers):
        for p in range(2):
            k, v = o.read_kv(l, p)
            assert np.all(k.view(np.uint32) & 0xFFFF == 0) and np.all(v.view(np.uint32) & 0xFFFF == 0)
            assert np.any(k != 0) and np.any(v != 0)


def test_gqa_equals_mha_with_repeated_kv_heads(oracle_lib):
    """Grouped-query attention with each KV head shared by a group of query heads
    is multi-head attention whose K/V projections repeat per group."""
    import dataclasses
    g = hp.SMALL_GQA
    m = dataclasses.replace(g, name="as-mha", n_kv_heads=g.n_q_heads)
    w = hp.shaped_weights(g, seed=9)
    wm = dict(w)
    rep = g.n_q_heads // g.n_kv_heads
    for l in range(g.n_layers):
        for nm in ("wk", "wv"):
            t = w[f"l{l}.{nm}"].reshape(g.n_kv_heads, g.head_dim, g.hidden)
            wm[f"l{l}.{nm}"] = t.repeat_interleave(rep, dim=0).reshape(-1, g.hidden).contiguous()
    og, om = oracle_lib.Oracle(g, 8), oracle_lib.Oracle(m, 8)
    og.set_weights(w)
    om.set_weights(wm)
    for t, tok in enumerate([4, 77, 150, 9]):
        assert np.array_equal(og.forward_row(tok, t), om.forward_row(tok, t))


def test_thread_count_does_not_change_results(oracle_lib):
    s = hp.SMALL_GQA
    w = hp.shaped_weights(s, seed=10)
    a, b = oracle_lib.Oracle(s, 8, threads=1), oracle_lib.Oracle(s, 8, threads=4)
    a.set_weights(w)
    b.set_weights(w)
    for t, tok in enumerate([1, 2, 3]):
        assert np.array_equal(a.forward_row(tok, t), b.forward_row(tok, t))


def test_weight_generator_moments_and_checksum():
    x = si.normal_tensor(0, 1, 1 << 20)
    assert abs(float(x.mean())) < 1e-4 and abs(float(x.std()) - 0.02) < 1e-4
    k = float(((x / 0.02) ** 4).mean())
    assert abs(k - 3.0) < 0.05                       # Gaussian kurtosis
    # integer stage of the generator is bit-exact everywhere: torch path == pure-Python path
    key = si.tensor_key(0, 1)
    idx = torch.arange(0, 5, dtype=torch.int64)
    got = [int(v) & si._M64 for v in si._mix64_t(idx + si._s64(key))]
    assert got == [si.mix64((key + i) & si._M64) for i in range(5)]
    assert si.mix64(0) == 0xE220A8397B1DCDAF          # splitmix64's first output for seed 0
    b = si.normal_tensor(0, 1, 1024, dtype=torch.bfloat16)
    assert torch.equal(b, x[:1024].bfloat16())
    m = si.random_mask(32, 32, 2)
    assert m.sum() == 32 and m[:4].sum() == 0 and m[-4:].sum() == 0
    assert list(np.nonzero(si.tiny_mask())[0]) == [2, 5]
    ids = si.uniform_ids(1, 4096, 1000)
    assert ids.min() >= 0 and ids.max() < 1000 and len(set(ids.tolist())) > 900
