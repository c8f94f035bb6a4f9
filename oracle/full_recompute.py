"""Brute-force, cache-free recompute of the decoder over a whole sequence (fp64).

TEST INFRASTRUCTURE ONLY.  A second statement of the same model as
``oracle.c``, independent of it: all positions at once, an explicit n x n score
matrix with -inf above the diagonal, no KV cache, numpy float64 throughout.
The CPU tests require the cached, token-by-token C oracle to agree with this
routine, which is the invariant "incremental decode equals full recompute"
(the paper's Alg. 1 produces one token per step from cached state; Sec. III-A
lists the operators).  Meant for tiny models only.

``weights`` is a dict with keys ``tok_emb`` [V,d], ``final_norm`` [d],
``lm_head`` [V,d] and ``layers``: a list of dicts with ``attn_norm`` [d],
``wq``/``wk``/``wv``/``wo`` [d,d], ``ffn_norm`` [d], ``w_gate``/``w_up`` [F,d],
``w_down`` [d,F]; every linear map is row-major [out, in] (y = W x).
"""
import numpy as np


def _rmsnorm_rows(X, g, eps):
    r = np.mean(X * X, axis=1, keepdims=True)
    return X / np.sqrt(r + eps) * g[None, :]


def _rope_rows(X, n_heads, head_dim, theta):
    """Rotate-half RoPE for rows at positions 0..n-1."""
    n = X.shape[0]
    half = head_dim // 2
    Xh = X.reshape(n, n_heads, head_dim).copy()
    j = np.arange(half, dtype=np.float64)
    inv_freq = np.float64(theta) ** (-2.0 * j / head_dim)
    phi = np.arange(n, dtype=np.float64)[:, None] * inv_freq[None, :]      # [n, half]
    c = np.cos(phi)[:, None, :]
    s = np.sin(phi)[:, None, :]
    lo = Xh[:, :, :half]
    hi = Xh[:, :, half:]
    out = np.empty_like(Xh)
    out[:, :, :half] = lo * c - hi * s
    out[:, :, half:] = hi * c + lo * s
    return out.reshape(n, n_heads * head_dim)


def forward_full(cfg, weights, tokens):
    """Logits [n, vocab] and final residual stream [n, d] for every position."""
    d, H, dh = cfg["d_model"], cfg["n_heads"], cfg["head_dim"]
    eps, theta = float(cfg["rms_eps"]), float(cfg["rope_theta"])
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    tokens = np.asarray(tokens, dtype=np.int64)
    n = tokens.shape[0]
    X = f64(weights["tok_emb"])[tokens]                                   # [n, d]
    causal = np.triu(np.ones((n, n), dtype=bool), k=1)                      # True above diagonal
    for L in weights["layers"]:
        A = _rmsnorm_rows(X, f64(L["attn_norm"]), eps)
        Q = _rope_rows(A @ f64(L["wq"]).T, H, dh, theta)
        K = _rope_rows(A @ f64(L["wk"]).T, H, dh, theta)
        Vv = A @ f64(L["wv"]).T
        O = np.empty_like(X)
        for h in range(H):
            sl = slice(h * dh, (h + 1) * dh)
            S = (Q[:, sl] @ K[:, sl].T) / np.sqrt(np.float64(dh))
            S = np.where(causal, -np.inf, S)
            S = S - S.max(axis=1, keepdims=True)
            P = np.exp(S)
            P = P / P.sum(axis=1, keepdims=True)
            O[:, sl] = P @ Vv[:, sl]
        X = X + O @ f64(L["wo"]).T
        B = _rmsnorm_rows(X, f64(L["ffn_norm"]), eps)
        G = B @ f64(L["w_gate"]).T
        U = B @ f64(L["w_up"]).T
        M = G / (1.0 + np.exp(-G)) * U
        X = X + M @ f64(L["w_down"]).T
    logits = _rmsnorm_rows(X, f64(weights["final_norm"]), eps) @ f64(weights["lm_head"]).T
    return logits, X
