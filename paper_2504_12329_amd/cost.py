"""Closed-form work counts of the decoder step (host arithmetic only, used for rooflines).

Matmul FLOPs follow Appendix A of the paper (which assumes multi-head attention, h = n*d) made
GQA-aware; with n_kv_heads == n_q_heads they reduce to that appendix's matmul terms.  Bytes
are the algorithmic HBM traffic of one decode step: every weight once, the KV cache once.
"""


def layer_matmul_params(cfg):
    h, d = cfg["hidden"], cfg["head_dim"]
    nq, nkv, I = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["intermediate"]
    return 2 * h * nq * d + 2 * h * nkv * d + 3 * h * I


def decode_flops_layer(cfg, s):
    """Matmul FLOPs of one layer for one new token attending to s keys."""
    nq, d = cfg["n_q_heads"], cfg["head_dim"]
    return 2 * layer_matmul_params(cfg) + 4 * nq * d * s


def prefill_flops_layer(cfg, m, kv0=0, causal=True):
    """Matmul FLOPs of one layer for m new tokens on top of kv0 cached ones."""
    nq, d = cfg["n_q_heads"], cfg["head_dim"]
    keys = m * kv0 + (m * (m + 1) // 2 if causal else m * m)
    return 2 * m * layer_matmul_params(cfg) + 4 * nq * d * keys


def prefill_flops(cfg, m, kv0=0):
    """Whole-model catch-up pass: all layers plus the LM head for the last row only."""
    return cfg["n_layers"] * prefill_flops_layer(cfg, m, kv0) + 2 * cfg["hidden"] * cfg["vocab"]


def weight_bytes(cfg):
    """bf16 bytes of every matrix a decode step streams (LM head once; tied embedding row is negligible)."""
    return 2 * (cfg["n_layers"] * layer_matmul_params(cfg) + cfg["vocab"] * cfg["hidden"])


def kv_bytes_per_position(cfg):
    return cfg["n_layers"] * 2 * cfg["n_kv_heads"] * cfg["head_dim"] * 2


def decode_bytes(cfg, t):
    """Algorithmic HBM bytes of one decode step whose query attends to t keys (the new one included)."""
    return weight_bytes(cfg) + t * kv_bytes_per_position(cfg)
