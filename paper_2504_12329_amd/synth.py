"""Seeded synthetic inputs: model shapes, random-init weights, prompts and trigger bitmaps.

This module serves both the HIP path and the tests' CPU oracle and therefore holds none of
the method's arithmetic: it only draws random numbers, rounds them to bf16 once, and lays
tensors out.  The shapes are those of the Qwen-2.5 / DeepSeek-R1-Distill models the paper
evaluates (1.5B, 7B, 32B; Table 2) plus a tiny pair for exhaustive checking.
"""
import hashlib

import numpy as np
import torch

SHAPES = {
    # name: n_layers, hidden, n_q_heads, n_kv_heads, head_dim, intermediate, vocab, tied
    "tiny_small": (2, 256, 4, 2, 64, 688, 1024, 0),
    "tiny_large": (4, 256, 4, 2, 64, 688, 1024, 0),
    "qwen1p5b": (28, 1536, 12, 2, 128, 8960, 151936, 1),
    "qwen7b": (28, 3584, 28, 4, 128, 18944, 152064, 0),
    "qwen32b": (64, 5120, 40, 8, 128, 27648, 152064, 0),
}


def model_config(name, max_seq, max_chunk=None, n_layers=None):
    L, h, nq, nkv, d, I, V, tied = SHAPES[name]
    return dict(n_layers=n_layers or L, hidden=h, n_q_heads=nq, n_kv_heads=nkv, head_dim=d,
                intermediate=I, vocab=V, rms_eps=1e-6, rope_theta=1e6, tie_embeddings=tied,
                qkv_bias=1, max_seq=int(max_seq), max_chunk=int(max_chunk or min(max_seq, 4096)))


def _seed_for(seed, name, layer):
    hsh = hashlib.sha256(f"{seed}/{name}/{layer}".encode()).digest()
    return int.from_bytes(hsh[:7], "little")


def _normal(shape, seed, name, layer, device, mean=0.0, std=0.02):
    g = torch.Generator(device=device)
    g.manual_seed(_seed_for(seed, name, layer))
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(mean, std, generator=g)
    return t.to(torch.bfloat16)          # rounded to nearest-even once; both sides get these bits


def make_layer(cfg, seed, layer, device="cpu"):
    """bf16 tensors of one decoder layer in the GPU library's layouts."""
    h, d = cfg["hidden"], cfg["head_dim"]
    nq, nkv, I = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["intermediate"]
    qkv = (nq + 2 * nkv) * d
    return dict(
        wqkv=_normal((qkv, h), seed, "wqkv", layer, device),          # rows: q heads, then k heads, then v heads
        bqkv=_normal((qkv,), seed, "bqkv", layer, device),
        wo=_normal((h, nq * d), seed, "wo", layer, device),
        w_gate_up=_normal((2 * I, h), seed, "w_gate_up", layer, device),  # rows: gate [0,I), up [I,2I)
        w_down=_normal((h, I), seed, "w_down", layer, device),
        norm_attn=_normal((h,), seed, "norm_attn", layer, device, mean=1.0),
        norm_mlp=_normal((h,), seed, "norm_mlp", layer, device, mean=1.0),
    )


def make_weights(cfg, seed, device="cpu"):
    """All weights of a model: matrices, embeddings and biases ~ N(0, 0.02), norm gains ~ 1 + N(0, 0.02)."""
    w = dict(
        embed=_normal((cfg["vocab"], cfg["hidden"]), seed, "embed", -1, device),
        final_norm=_normal((cfg["hidden"],), seed, "final_norm", -1, device, mean=1.0),
        layers=[make_layer(cfg, seed, l, device) for l in range(cfg["n_layers"])],
    )
    w["lm_head"] = None if cfg["tie_embeddings"] else _normal((cfg["vocab"], cfg["hidden"]), seed, "lm_head", -1, device)
    return w


def oracle_views(cfg, w):
    """The same bits widened to fp32 numpy arrays and split into the oracle's per-matrix naming."""
    d, nq, nkv, I = cfg["head_dim"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["intermediate"]
    f = lambda t: t.detach().to("cpu").float().numpy()
    out = dict(embed=f(w["embed"]), final_norm=f(w["final_norm"]),
               lm_head=None if w["lm_head"] is None else f(w["lm_head"]))
    for k in ("wq", "wk", "wv", "bq", "bk", "bv", "wo", "wg", "wu", "wd", "norm_attn", "norm_mlp"):
        out[k] = []
    a, b = nq * d, (nq + nkv) * d
    for lw in w["layers"]:
        wqkv, bqkv, gu = f(lw["wqkv"]), f(lw["bqkv"]), f(lw["w_gate_up"])
        out["wq"].append(wqkv[:a]); out["wk"].append(wqkv[a:b]); out["wv"].append(wqkv[b:])
        out["bq"].append(bqkv[:a]); out["bk"].append(bqkv[a:b]); out["bv"].append(bqkv[b:])
        out["wg"].append(gu[:I]); out["wu"].append(gu[I:])
        out["wo"].append(f(lw["wo"])); out["wd"].append(f(lw["w_down"]))
        out["norm_attn"].append(f(lw["norm_attn"])); out["norm_mlp"].append(f(lw["norm_mlp"]))
    return out


def oracle_config(cfg):
    keys = ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "intermediate", "vocab",
            "rms_eps", "rope_theta", "qkv_bias", "max_seq")
    return {k: cfg[k] for k in keys}


def make_prompt(n, vocab, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.integers(0, vocab, size=n, dtype=np.int32)


def modulo_bitmap(vocab, modulus):
    """Bitmap (uint32 words, bit id&31 of word id>>5) of the token ids divisible by `modulus`."""
    ids = np.arange(0, vocab, modulus, dtype=np.int64)
    bm = np.zeros((vocab + 31) // 32, dtype=np.uint32)
    np.bitwise_or.at(bm, ids >> 5, (np.uint32(1) << (ids & 31).astype(np.uint32)))
    return bm
