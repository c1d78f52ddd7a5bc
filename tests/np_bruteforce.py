"""Brute-force fp64 numpy evaluation of a whole token sequence, used only to pin the C oracle.

No cache, no per-position loop: every layer is a handful of dense matrix products over all T
positions with an explicit causal mask, written in the textbook matrix form
(softmax(Q K^T / sqrt(d) + mask) V, x*cos + rotate_half(x)*sin).  It is structured as
differently from the oracle's per-token loop as the mathematics allows.
"""
import numpy as np


def _rms(X, g, eps):
    return X / np.sqrt((X * X).mean(axis=-1, keepdims=True) + eps) * g


def _rotate_half(X):
    half = X.shape[-1] // 2
    return np.concatenate([-X[..., half:], X[..., :half]], axis=-1)


def _rope(X, positions, theta):
    """X [T][heads][d]"""
    d = X.shape[-1]
    inv = theta ** (-np.arange(0, d, 2, dtype=np.float64) / d)          # d/2 frequencies
    ang = np.outer(positions.astype(np.float64), inv)                   # [T][d/2]
    cos = np.concatenate([np.cos(ang), np.cos(ang)], axis=-1)[:, None, :]
    sin = np.concatenate([np.sin(ang), np.sin(ang)], axis=-1)[:, None, :]
    return X * cos + _rotate_half(X) * sin


def forward_all(cfg, w, tokens, pos0=0):
    """Logits [T][vocab] (fp64) of every position of `tokens`, positions pos0..pos0+T-1, no prior context."""
    f = lambda a: np.asarray(a, dtype=np.float64)
    T = len(tokens)
    h, d, nq, nkv = cfg["hidden"], cfg["head_dim"], cfg["n_q_heads"], cfg["n_kv_heads"]
    G = nq // nkv
    X = f(w["embed"])[np.asarray(tokens)]
    pos = np.arange(pos0, pos0 + T)
    mask = np.where(np.arange(T)[None, :] > np.arange(T)[:, None], -np.inf, 0.0)
    for l in range(cfg["n_layers"]):
        Y = _rms(X, f(w["norm_attn"][l]), cfg["rms_eps"])
        Q = Y @ f(w["wq"][l]).T
        K = Y @ f(w["wk"][l]).T
        V = Y @ f(w["wv"][l]).T
        if cfg.get("qkv_bias", 1):
            Q, K, V = Q + f(w["bq"][l]), K + f(w["bk"][l]), V + f(w["bv"][l])
        Q = _rope(Q.reshape(T, nq, d), pos, cfg["rope_theta"])
        K = _rope(K.reshape(T, nkv, d), pos, cfg["rope_theta"])
        V = V.reshape(T, nkv, d)
        K = np.repeat(K, G, axis=1)          # kv head g serves query heads g*G .. g*G+G-1
        V = np.repeat(V, G, axis=1)
        S = np.einsum("ihd,jhd->hij", Q, K) / np.sqrt(d) + mask[None]
        S = S - S.max(axis=-1, keepdims=True)
        Pm = np.exp(S)
        Pm = Pm / Pm.sum(axis=-1, keepdims=True)
        O = np.einsum("hij,jhd->ihd", Pm, V).reshape(T, nq * d)
        X = X + O @ f(w["wo"][l]).T
        Y = _rms(X, f(w["norm_mlp"][l]), cfg["rms_eps"])
        Gt = Y @ f(w["wg"][l]).T
        U = Y @ f(w["wu"][l]).T
        X = X + ((Gt / (1.0 + np.exp(-Gt))) * U) @ f(w["wd"][l]).T
    Y = _rms(X, f(w["final_norm"]), cfg["rms_eps"])
    head = w["embed"] if w.get("lm_head") is None else w["lm_head"]
    return Y @ f(head).T
