"""Pins of the CPU oracle against things other than itself.

The paper prints no worked numeric example, so nothing in it fixes a value;
each operator is pinned to what the mathematics fixes (closed forms,
invariants, special cases that collapse to a library fp64 matmul) and the
whole model to (i) an independent brute-force recompute over the full
sequence, (ii) causality, (iii) degenerate weight settings, (iv) a head
permutation symmetry.  All CPU; a plausible slip in oracle.c (dropped term,
wrong sign/index, transposed operand, wrong pairing, off-by-one in the causal
range) fails at least one test here.
"""
import json
import os

import numpy as np
import pytest

from oracle import full_recompute
from paper_2604_23467_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
EPS = float(np.float32(1e-5))      # the configuration carries eps as a C float


def both(fn):
    return pytest.mark.parametrize("prec", ["f32", "f64"])(fn)


def get(prec, oracle32, oracle64):
    return oracle32 if prec == "f32" else oracle64


def tol(prec, t32, t64):
    return t32 if prec == "f32" else t64


# ---------------------------------------------------------------- fp16 decode
def test_half_to_float_all_bit_patterns(oracle32):
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)          # library conversion
    got = np.array([oracle32.half_to_float(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def test_fp16_weights_are_upcast_exactly(oracle64):
    rng = np.random.default_rng(1)
    W = (0.02 * rng.standard_normal((7, 24))).astype(np.float16)
    x = rng.standard_normal(24)
    y = oracle64.matvec(W, x)
    assert np.allclose(y, W.astype(np.float64) @ x, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- RMSNorm
@both
def test_rmsnorm_constant_vector_closed_form(prec, oracle32, oracle64):
    o = get(prec, oracle32, oracle64)
    n, c, eps = 96, 0.37, EPS
    out = o.rmsnorm(np.full(n, c), np.ones(n, dtype=np.float32), eps)
    assert np.allclose(out, c / np.sqrt(c * c + eps), rtol=tol(prec, 1e-6, 1e-13), atol=0)


@both
def test_rmsnorm_mean_square_and_gain(prec, oracle32, oracle64):
    o = get(prec, oracle32, oracle64)
    rng = np.random.default_rng(2)
    n, eps = 200, EPS
    x = rng.standard_normal(n) * 3.0
    r = np.mean(x * x)
    out1 = o.rmsnorm(x, np.ones(n, dtype=np.float32), eps).astype(np.float64)
    # mean(out^2) = r / (r + eps) : eps sits inside the root, added to the mean square
    assert np.isclose(np.mean(out1 * out1), r / (r + eps), rtol=tol(prec, 1e-5, 1e-12))
    # no mean subtraction: a shifted vector keeps its sign pattern scaled by one factor
    assert np.allclose(out1 / x, out1[0] / x[0], rtol=tol(prec, 1e-5, 1e-12))
    g = (1.0 + 0.5 * rng.standard_normal(n)).astype(np.float32)
    outg = o.rmsnorm(x, g, eps).astype(np.float64)
    assert np.allclose(outg, out1 * g.astype(np.float64), rtol=tol(prec, 1e-5, 1e-12), atol=1e-30)
    # eps matters when the vector is tiny: x = 1e-3 * ones, r = 1e-6 < eps
    small = o.rmsnorm(np.full(n, 1e-3), np.ones(n, dtype=np.float32), eps)
    assert np.allclose(small, 1e-3 / np.sqrt(1e-6 + eps), rtol=tol(prec, 1e-5, 1e-12))


# ---------------------------------------------------------------- linear maps
@both
def test_matvec_matches_library_fp64_matmul_nonsquare(prec, oracle32, oracle64):
    o = get(prec, oracle32, oracle64)
    rng = np.random.default_rng(3)
    for n_out, n_in in [(5, 9), (33, 17), (64, 257)]:
        W = rng.standard_normal((n_out, n_in)).astype(np.float32)
        x = rng.standard_normal(n_in)
        y = o.matvec(W, x)
        ref = W.astype(np.float64) @ np.asarray(x, dtype=o.real).astype(np.float64)
        assert y.shape == (n_out,)
        assert np.allclose(y, ref, rtol=0, atol=tol(prec, 2e-5, 1e-12))
    # a one-hot input picks a column (row-major [out, in], y = W x, not W^T x)
    W = rng.standard_normal((4, 6)).astype(np.float32)
    e = np.zeros(6); e[4] = 1.0
    assert np.allclose(o.matvec(W, e), W[:, 4], atol=1e-7)


# ---------------------------------------------------------------- RoPE
@both
def test_rope_pairing_on_a_unit_vector(prec, oracle32, oracle64):
    """Reading: rotate-half.  head_dim 4, pos 1: pair (0,2) turns by 1 rad,
    pair (1,3) by 1/theta^(1/2) = 0.01 rad.  Values from tests/golden/rope_unit.json."""
    o = get(prec, oracle32, oracle64)
    gold = json.load(open(os.path.join(GOLDEN, "rope_unit.json")))
    for case in gold["cases"]:
        got = o.rope(np.array(case["x"], dtype=np.float64), 1, 4, case["pos"], gold["theta"])
        assert np.allclose(got, case["y"], rtol=0, atol=tol(prec, 1e-6, 1e-12)), case


@both
def test_rope_invariants(prec, oracle32, oracle64):
    o = get(prec, oracle32, oracle64)
    rng = np.random.default_rng(4)
    H, dh, theta = 3, 16, 10000.0
    x = rng.standard_normal(H * dh)
    t = tol(prec, 3e-6, 1e-12)
    # position 0 is the identity
    assert np.array_equal(o.rope(x, H, dh, 0, theta), x.astype(o.real))
    # each (j, j+dh/2) pair keeps its norm
    y = o.rope(x, H, dh, 37, theta).astype(np.float64).reshape(H, dh)
    xr = x.reshape(H, dh)
    n_in = xr[:, :dh // 2] ** 2 + xr[:, dh // 2:] ** 2
    n_out = y[:, :dh // 2] ** 2 + y[:, dh // 2:] ** 2
    assert np.allclose(n_in, n_out, rtol=t * 10)
    # rotations compose additively
    ab = o.rope(o.rope(x, H, dh, 5, theta), H, dh, 11, theta)
    assert np.allclose(ab, o.rope(x, H, dh, 16, theta), atol=t * 10)
    # <rope(q,m), rope(k,n)> per head depends on m - n only
    q, k = rng.standard_normal(H * dh), rng.standard_normal(H * dh)
    def dots(m, n):
        a = o.rope(q, H, dh, m, theta).astype(np.float64).reshape(H, dh)
        b = o.rope(k, H, dh, n, theta).astype(np.float64).reshape(H, dh)
        return (a * b).sum(axis=1)
    assert np.allclose(dots(9, 4), dots(25, 20), atol=t * 50)
    assert not np.allclose(dots(9, 4), dots(9, 5), atol=1e-3)
    # frequency ladder: component j of a unit vector turns by pos * theta^(-2j/dh)
    for j in (0, 1, 5, 7):
        e = np.zeros(dh); e[j] = 1.0
        r = o.rope(e, 1, dh, 3, theta)
        phi = 3.0 * theta ** (-2.0 * j / dh)
        assert np.isclose(r[j], np.cos(phi), atol=t) and np.isclose(r[j + dh // 2], np.sin(phi), atol=t)


# ---------------------------------------------------------------- attention
@both
def test_attention_head_special_cases(prec, oracle32, oracle64):
    o = get(prec, oracle32, oracle64)
    rng = np.random.default_rng(5)
    dh, n = 16, 7
    K, V = rng.standard_normal((n, dh)), rng.standard_normal((n, dh))
    q = rng.standard_normal(dh)
    t = tol(prec, 2e-6, 1e-13)
    out, w = o.attention_head(q, K, V)
    assert np.isclose(w.sum(), 1.0, atol=t) and (w > 0).all()
    # definition with the 1/sqrt(dh) scale, in fp64
    s = K @ q / np.sqrt(dh)
    p = np.exp(s - s.max()); p /= p.sum()
    assert np.allclose(w, p, atol=t) and np.allclose(out, p @ V, atol=t * 10)
    # zero query -> uniform weights -> mean of the value rows
    out0, w0 = o.attention_head(np.zeros(dh), K, V)
    assert np.allclose(w0, 1.0 / n, atol=t) and np.allclose(out0, V.mean(axis=0), atol=t * 10)
    # a single key returns its value row exactly
    out1, w1 = o.attention_head(q, K[:1], V[:1])
    assert w1[0] == 1.0 and np.array_equal(out1, V[0].astype(o.real))
    # shift invariance: adding c*q/|q|^2-aligned constant to all scores changes nothing
    big, _ = o.attention_head(q * 40.0, K, V)      # large scores: max-subtraction keeps it finite
    assert np.isfinite(big).all()
    s2 = K @ (q * 40.0) / np.sqrt(dh)
    p2 = np.exp(s2 - s2.max()); p2 /= p2.sum()
    assert np.allclose(big, p2 @ V, atol=tol(prec, 2e-4, 1e-11))


# ---------------------------------------------------------------- SwiGLU, argmax
@both
def test_swiglu_closed_forms(prec, oracle32, oracle64):
    o = get(prec, oracle32, oracle64)
    g = np.array([0.0, 1.0, -1.0, 30.0, -30.0, 2.5])
    u = np.array([3.0, 2.0, 2.0, 1.5, 1.5, -4.0])
    m = o.swiglu(g, u).astype(np.float64)
    assert m[0] == 0.0                                            # silu(0) = 0
    assert np.isclose(m[1], 2.0 / (1.0 + np.exp(-1.0)), rtol=1e-6)   # silu(1)*2
    assert np.isclose(m[2], -2.0 / (1.0 + np.exp(1.0)), rtol=1e-6)   # silu(-1)*2
    assert np.isclose(m[3], 45.0, rtol=1e-6)                       # silu(z) -> z
    assert abs(m[4]) < 1e-10                                       # silu(z) -> 0
    assert np.isclose(m[5], 2.5 / (1.0 + np.exp(-2.5)) * -4.0, rtol=1e-6)


def test_argmax_brute_force_and_ties(oracle32):
    rng = np.random.default_rng(6)
    for _ in range(20):
        v = rng.standard_normal(50).astype(np.float32)
        assert oracle32.argmax(v) == int(np.argmax(v))
    v = np.zeros(10, dtype=np.float32)
    assert oracle32.argmax(v) == 0
    v[[3, 7]] = 2.0
    assert oracle32.argmax(v) == 3            # lowest index among equal maxima
    v[9] = 5.0
    assert oracle32.argmax(v) == 9


# ---------------------------------------------------------------- whole model
def _run_cached(o, cfg, w, tokens):
    m = o.model(cfg, w)
    logits, hidden, toks = [], [], []
    for t in tokens:
        nt, lg, hd = m.step(int(t))
        logits.append(lg.copy()); hidden.append(hd.copy()); toks.append(nt)
    m.close()
    return np.array(logits), np.array(hidden), toks


def _small_cfg():
    return wl.custom_cfg(n_layers=2, n_heads=3, head_dim=8, ffn_hidden=40, vocab=50, max_seq=16)


@both
def test_cached_decode_equals_full_recompute(prec, oracle32, oracle64):
    o = get(prec, oracle32, oracle64)
    cfg = _small_cfg()
    w = wl.make_weights_numpy(cfg, seed=11, gain_jitter=0.3, emb_std=1.0)
    for L in w["layers"]:                       # O(1) activations so every term matters
        for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            L[k] *= 12.0
    tokens = wl.make_tokens(9, cfg["vocab"], seed=3)
    logits, hidden, _ = _run_cached(o, cfg, w, tokens)
    ref_logits, ref_hidden = full_recompute.forward_full(cfg, w, tokens)
    t = tol(prec, 2e-4, 1e-10)
    assert np.abs(hidden - ref_hidden).max() < t * max(1.0, np.abs(ref_hidden).max())
    assert np.abs(logits - ref_logits).max() < t * max(1.0, np.abs(ref_logits).max())


def test_tiny_config_cached_equals_full_recompute_fp32(oracle32):
    """BASELINE config 1 shape: fp32 oracle vs the fp64 brute force, <= 1e-5."""
    cfg = wl.tiny_cfg(max_seq=32)
    w = wl.make_weights_numpy(cfg, seed=0)
    tokens = wl.make_tokens(10, cfg["vocab"], seed=0)
    logits, hidden, _ = _run_cached(oracle32, cfg, w, tokens)
    ref_logits, ref_hidden = full_recompute.forward_full(cfg, w, tokens)
    assert np.abs(logits - ref_logits).max() < 1e-5
    assert np.abs(hidden - ref_hidden).max() < 1e-5


def test_fp32_oracle_close_to_fp64_oracle(oracle32, oracle64):
    cfg = wl.tiny_cfg(max_seq=32)
    w = wl.make_weights_numpy(cfg, seed=0)
    tokens = wl.make_tokens(12, cfg["vocab"], seed=1)
    l32, h32, t32 = _run_cached(oracle32, cfg, w, tokens)
    l64, h64, t64 = _run_cached(oracle64, cfg, w, tokens)
    assert np.abs(l32 - l64).max() < 1e-5 and np.abs(h32 - h64).max() < 1e-5


def test_causality(oracle64):
    cfg = _small_cfg()
    w = wl.make_weights_numpy(cfg, seed=12, emb_std=1.0)
    for L in w["layers"]:
        for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            L[k] *= 10.0
    a = wl.make_tokens(8, cfg["vocab"], seed=4)
    b = a.copy(); b[5:] = (b[5:] + 7) % cfg["vocab"]
    la, _, _ = _run_cached(oracle64, cfg, w, a)
    lb, _, _ = _run_cached(oracle64, cfg, w, b)
    assert np.array_equal(la[:5], lb[:5])
    assert np.abs(la[5:] - lb[5:]).max() > 1e-3
    # and the context does matter: same last token, different history
    c = a.copy(); c[0] = (c[0] + 1) % cfg["vocab"]
    lc, _, _ = _run_cached(oracle64, cfg, w, c)
    assert np.abs(la[7] - lc[7]).max() > 1e-6


def test_zero_output_projections_make_logits_context_free(oracle64):
    cfg = _small_cfg()
    w = wl.make_weights_numpy(cfg, seed=13, gain_jitter=0.2, emb_std=1.0)
    for L in w["layers"]:
        L["wo"][:] = 0.0
        L["w_down"][:] = 0.0
    tokens = wl.make_tokens(6, cfg["vocab"], seed=5)
    logits, hidden, _ = _run_cached(oracle64, cfg, w, tokens)
    E = w["tok_emb"].astype(np.float64)
    for p, t in enumerate(tokens):
        x = E[t]
        a = x / np.sqrt(np.mean(x * x) + EPS) * w["final_norm"].astype(np.float64)
        assert np.allclose(hidden[p], x, atol=1e-14)
        assert np.allclose(logits[p], w["lm_head"].astype(np.float64) @ a, atol=1e-12)


def test_first_position_layer_reduces_to_gemv_chain(oracle64):
    """At p = 0 there is one key, softmax = 1, RoPE = identity: one layer is
    x + Wo Wv a followed by the FFN -- pure library matmuls in fp64."""
    cfg = wl.custom_cfg(n_layers=1, n_heads=2, head_dim=8, ffn_hidden=24, vocab=30, max_seq=4)
    w = wl.make_weights_numpy(cfg, seed=14, gain_jitter=0.2, emb_std=1.0)
    L = {k: v.astype(np.float64) * (1.0 if k.endswith("norm") else 8.0) for k, v in w["layers"][0].items()}
    for k in L:
        w["layers"][0][k] = L[k].astype(np.float32)
        L[k] = w["layers"][0][k].astype(np.float64)
    eps = EPS
    rn = lambda x, g: x / np.sqrt(np.mean(x * x) + eps) * g
    tok = 7
    x = w["tok_emb"][tok].astype(np.float64)
    x = x + L["wo"] @ (L["wv"] @ rn(x, L["attn_norm"]))
    b = rn(x, L["ffn_norm"])
    g, u = L["w_gate"] @ b, L["w_up"] @ b
    x = x + L["w_down"] @ (g / (1 + np.exp(-g)) * u)
    ref = w["lm_head"].astype(np.float64) @ rn(x, w["final_norm"].astype(np.float64))
    m = oracle64.model(cfg, w)
    nt, logits, hidden = m.step(tok)
    assert np.allclose(hidden, x, atol=1e-11) and np.allclose(logits, ref, atol=1e-11)
    assert nt == int(np.argmax(ref))


def test_head_permutation_leaves_logits_unchanged(oracle64):
    cfg = _small_cfg()
    w = wl.make_weights_numpy(cfg, seed=15, emb_std=1.0)
    for L in w["layers"]:
        for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
            L[k] *= 10.0
    H, dh = cfg["n_heads"], cfg["head_dim"]
    perm = np.array([2, 0, 1])
    idx = (perm[:, None] * dh + np.arange(dh)[None, :]).reshape(-1)
    w2 = {k: v for k, v in w.items() if k != "layers"}
    w2["layers"] = []
    for L in w["layers"]:
        L2 = dict(L)
        for k in ("wq", "wk", "wv"):
            L2[k] = np.ascontiguousarray(L[k][idx, :])
        L2["wo"] = np.ascontiguousarray(L["wo"][:, idx])
        w2["layers"].append(L2)
    tokens = wl.make_tokens(7, cfg["vocab"], seed=6)
    la, _, _ = _run_cached(oracle64, cfg, w, tokens)
    lb, _, _ = _run_cached(oracle64, cfg, w2, tokens)
    assert np.allclose(la, lb, atol=1e-11)


def test_kv_cache_holds_rotated_keys_and_plain_values(oracle64):
    cfg = _small_cfg()
    w = wl.make_weights_numpy(cfg, seed=16, emb_std=1.0)
    tokens = wl.make_tokens(4, cfg["vocab"], seed=7)
    m = oracle64.model(cfg, w)
    for t in tokens:
        m.step(int(t))
    assert m.pos == 4
    E = w["tok_emb"].astype(np.float64)
    L0 = w["layers"][0]
    for p, t in enumerate(tokens):                # layer 0 input is the embedding itself
        x = E[t]
        a = x / np.sqrt(np.mean(x * x) + EPS) * L0["attn_norm"].astype(np.float64)
        k = oracle64.rope(L0["wk"].astype(np.float64) @ a, cfg["n_heads"], cfg["head_dim"], p,
                          cfg["rope_theta"])
        v = L0["wv"].astype(np.float64) @ a
        assert np.allclose(m.kv(0, 0)[p], k, atol=1e-12)
        assert np.allclose(m.kv(0, 1)[p], v, atol=1e-12)
    m.close()


def test_model_rejects_bad_input(oracle32):
    cfg = _small_cfg()
    w = wl.make_weights_numpy(cfg, seed=17)
    m = oracle32.model(cfg, w)
    with pytest.raises(ValueError):
        m.step(cfg["vocab"])
    for _ in range(cfg["max_seq"]):
        m.step(1)
    with pytest.raises(ValueError):
        m.step(1)                                # cache full
    m.reset()
    assert m.pos == 0
    m.step(1)
    m.close()
    bad = dict(cfg); bad["head_dim"] = 7
    with pytest.raises(ValueError):
        oracle32.model(bad, w)


def test_tiny_config_matches_stored_oracle_run(oracle32):
    """Regression pin: tests/golden/tiny_config_run.json was written by
    tests/golden/make_tiny_golden.py, which calls only oracle/."""
    gold = json.load(open(os.path.join(GOLDEN, "tiny_config_run.json")))
    cfg = wl.tiny_cfg(max_seq=gold["max_seq"])
    w = wl.make_weights_numpy(cfg, seed=gold["weight_seed"])
    prompt = wl.make_tokens(gold["prompt_len"], cfg["vocab"], seed=gold["token_seed"])
    assert prompt.tolist() == gold["prompt"]
    m = oracle32.model(cfg, w)
    t, logits, _ = m.prefill(prompt)
    toks, sums = [t], [float(np.abs(logits).sum())]
    for _ in range(gold["decode_steps"]):
        t, logits, _ = m.step(t)
        toks.append(t); sums.append(float(np.abs(logits).sum()))
    m.close()
    assert toks == gold["tokens"]
    assert np.allclose(sums, gold["logit_abs_sums"], rtol=1e-5)
