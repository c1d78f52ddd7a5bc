"""Pins of the CPU oracle against things other than itself: closed forms, invariants, textbook
special cases and a brute-force fp64 numpy evaluation of the whole sequence.  CPU only."""
import math

import numpy as np
import pytest

from paper_2504_12329_amd import synth
from tests import np_bruteforce as bf


def _tiny(name="tiny_small", seed=1, max_seq=128, **over):
    cfg = synth.model_config(name, max_seq=max_seq)
    cfg.update(over)
    w = synth.make_weights(cfg, seed)
    return cfg, synth.oracle_views(cfg, w)


def _model(oracle_lib, cfg, ow):
    return oracle_lib.OracleModel(synth.oracle_config(cfg), ow)


# ---------------------------------------------------------------- primitives

def test_silu_closed_forms(oracle_lib):
    o = oracle_lib
    assert o.silu(0.0) == 0.0
    assert abs(o.silu(1.0) - 1.0 / (1.0 + math.exp(-1.0))) < 1e-7
    assert abs(o.silu(-1.0) + 1.0 / (1.0 + math.e)) < 1e-7
    for z in (0.3, 2.5, 7.0, 30.0):
        assert abs(o.silu(z) - o.silu(-z) - z) < 1e-6 * max(1.0, z)     # silu(z) - silu(-z) = z
    assert abs(o.silu(40.0) - 40.0) < 1e-5 and abs(o.silu(-40.0)) < 1e-12


def test_softmax_rows_sum_to_one_and_shift_invariance(oracle_lib):
    rng = np.random.default_rng(0)
    for n in (1, 2, 33, 257):
        s = rng.normal(0, 3, n).astype(np.float32)
        p = oracle_lib.softmax(s)
        assert abs(float(p.astype(np.float64).sum()) - 1.0) < 1e-6
        assert np.all(p >= 0)
        p2 = oracle_lib.softmax(s + np.float32(11.5))
        assert np.allclose(p, p2, atol=1e-6)
    # two-point closed form: softmax([a, b])[0] = 1 / (1 + e^(b-a)); large scores must not overflow
    p = oracle_lib.softmax(np.array([1000.0, 1001.0], dtype=np.float32))
    assert abs(p[0] - 1.0 / (1.0 + math.e)) < 1e-6
    assert np.allclose(oracle_lib.softmax(np.zeros(8, np.float32)), 1.0 / 8)


def test_rmsnorm_properties(oracle_lib):
    rng = np.random.default_rng(1)
    x = rng.normal(0, 2, 256).astype(np.float32)
    ones = np.ones(256, np.float32)
    y = oracle_lib.rmsnorm(x, ones, 0.0)
    assert abs(np.sqrt(np.mean(y.astype(np.float64) ** 2)) - 1.0) < 1e-6       # unit rms when g == 1
    y3 = oracle_lib.rmsnorm(3.0 * x, ones, 0.0)
    assert np.allclose(y, y3, atol=1e-6)                                       # scale invariance
    g = rng.normal(1, 0.1, 256).astype(np.float32)
    assert np.allclose(oracle_lib.rmsnorm(x, g, 0.0), y * g, atol=1e-6)        # gain multiplies
    # eps enters under the root next to the MEAN square: x = (1,1,1,1), eps = 3 -> 1/sqrt(1+3) = 0.5
    y = oracle_lib.rmsnorm(np.ones(4, np.float32), np.ones(4, np.float32), 3.0)
    assert np.allclose(y, 0.5, atol=1e-7)


def test_rope_closed_forms(oracle_lib):
    # d = 2 has the single frequency theta^0 = 1: a plain planar rotation by `pos` radians
    v = oracle_lib.rope(np.array([1.0, 0.0], np.float32), 1, 1e6)
    assert np.allclose(v, [math.cos(1.0), math.sin(1.0)], atol=1e-7)
    v = oracle_lib.rope(np.array([0.0, 1.0], np.float32), 3, 1e6)
    assert np.allclose(v, [-math.sin(3.0), math.cos(3.0)], atol=1e-7)
    # d = 4, theta = 100: pair (0,2) turns by pos*1, pair (1,3) by pos*100^(-2/4) = pos/10
    v = oracle_lib.rope(np.array([1.0, 1.0, 0.0, 0.0], np.float32), 5, 100.0)
    assert np.allclose(v, [math.cos(5.0), math.cos(0.5), math.sin(5.0), math.sin(0.5)], atol=1e-7)
    rng = np.random.default_rng(2)
    x = rng.normal(size=64).astype(np.float32)
    assert np.array_equal(oracle_lib.rope(x, 0, 1e6), x)                        # position 0 is the identity
    assert abs(np.linalg.norm(oracle_lib.rope(x, 777, 1e6)) - np.linalg.norm(x)) < 1e-5


def test_rope_scores_depend_on_relative_position_only(oracle_lib):
    rng = np.random.default_rng(3)
    q = rng.normal(size=128).astype(np.float32)
    k = rng.normal(size=128).astype(np.float32)
    base = float(np.dot(oracle_lib.rope(q, 17, 1e6).astype(np.float64), oracle_lib.rope(k, 5, 1e6)))
    moved = float(np.dot(oracle_lib.rope(q, 1017, 1e6).astype(np.float64), oracle_lib.rope(k, 1005, 1e6)))
    assert abs(base - moved) < 1e-4
    other = float(np.dot(oracle_lib.rope(q, 18, 1e6).astype(np.float64), oracle_lib.rope(k, 5, 1e6)))
    assert abs(base - other) > 1e-3                                             # and it does depend on the offset


def test_argmax_ties_and_nan(oracle_lib):
    assert oracle_lib.argmax(np.array([1, 5, 5, 2], np.float32)) == 1           # lowest index on ties
    assert oracle_lib.argmax(np.array([np.nan, 1, np.nan, 3, 3], np.float32)) == 3
    assert oracle_lib.argmax(np.array([np.nan, np.nan], np.float32)) == -1
    assert oracle_lib.argmax(np.array([-np.inf, -np.inf], np.float32)) == 0
    rng = np.random.default_rng(4)
    for _ in range(20):
        v = rng.integers(0, 7, 50).astype(np.float32)
        want = next(i for i in range(50) if v[i] == v.max())
        assert oracle_lib.argmax(v) == want


def _naive_attention(q, K, V, G):
    """Textbook softmax(q K^T / sqrt(d)) V in fp64, one head at a time."""
    nq, d = q.shape
    out = np.zeros((nq, d))
    for h in range(nq):
        g = h // G
        s = (K[:, g, :].astype(np.float64) @ q[h].astype(np.float64)) / math.sqrt(d)
        e = np.exp(s - s.max())
        out[h] = (e / e.sum()) @ V[:, g, :].astype(np.float64)
    return out


@pytest.mark.parametrize("nq,nkv,d,t", [(4, 2, 64, 1), (4, 2, 64, 37), (12, 2, 128, 65), (5, 1, 8, 9), (3, 3, 16, 20)])
def test_attention_matches_naive_softmax_qkv(oracle_lib, nq, nkv, d, t):
    rng = np.random.default_rng(nq * 1000 + t)
    q = rng.normal(size=(nq, d)).astype(np.float32)
    K = rng.normal(size=(t, nkv, d)).astype(np.float32)
    V = rng.normal(size=(t, nkv, d)).astype(np.float32)
    got = oracle_lib.attention(q, K, V)
    assert np.allclose(got, _naive_attention(q, K, V, nq // nkv), atol=2e-6)


def test_gqa_equals_mha_with_duplicated_kv_heads(oracle_lib):
    rng = np.random.default_rng(5)
    nq, nkv, d, t = 6, 2, 32, 25
    q = rng.normal(size=(nq, d)).astype(np.float32)
    K = rng.normal(size=(t, nkv, d)).astype(np.float32)
    V = rng.normal(size=(t, nkv, d)).astype(np.float32)
    gqa = oracle_lib.attention(q, K, V)
    mha = oracle_lib.attention(q, np.repeat(K, 3, axis=1), np.repeat(V, 3, axis=1))
    assert np.array_equal(gqa, mha)
    # a wrong head->group map (h % nkv instead of h // G) would give this instead:
    wrong = _naive_attention(q, np.tile(K, (1, 3, 1)), np.tile(V, (1, 3, 1)), 1)
    assert not np.allclose(gqa, wrong, atol=1e-3)


def test_attention_uniform_when_query_is_zero(oracle_lib):
    rng = np.random.default_rng(6)
    K = rng.normal(size=(11, 2, 16)).astype(np.float32)
    V = rng.normal(size=(11, 2, 16)).astype(np.float32)
    out = oracle_lib.attention(np.zeros((4, 16), np.float32), K, V)
    want = np.repeat(V.astype(np.float64).mean(axis=0), 2, axis=0)
    assert np.allclose(out, want, atol=1e-6)


# ---------------------------------------------------------------- whole model

@pytest.mark.parametrize("name,seed", [("tiny_small", 1), ("tiny_large", 2)])
def test_cached_decode_equals_full_causal_recompute(oracle_lib, name, seed):
    cfg, ow = _tiny(name, seed)
    toks = synth.make_prompt(24, cfg["vocab"], 3)
    m = _model(oracle_lib, cfg, ow)
    got = m.feed(toks, all_logits=True)                      # token by token with the cache
    want = bf.forward_all(cfg, ow, toks)                     # no cache, all positions at once, fp64
    scale = np.abs(want).max()
    assert np.abs(got - want).max() / scale < 1e-5
    assert m.kv_len == 24
    # the last position alone, after feeding a prefix first (cache carried across calls)
    m2 = _model(oracle_lib, cfg, ow)
    m2.feed(toks[:10])
    last = m2.feed(toks[10:])
    assert np.abs(last - want[-1]).max() / scale < 1e-5


def test_no_bias_and_mha_variants_match_bruteforce(oracle_lib):
    cfg, ow = _tiny("tiny_small", 7, qkv_bias=0)
    toks = synth.make_prompt(9, cfg["vocab"], 8)
    got = _model(oracle_lib, cfg, ow).feed(toks, all_logits=True)
    want = bf.forward_all(cfg, ow, toks)
    assert np.abs(got - want).max() / np.abs(want).max() < 1e-5
    with_bias = dict(cfg, qkv_bias=1)
    assert np.abs(bf.forward_all(with_bias, ow, toks) - want).max() > 1e-4      # the bias is not a no-op


@pytest.mark.parametrize("split", [1, 7, 15])
def test_chunked_prefill_equals_one_pass_equals_decode(oracle_lib, split):
    cfg, ow = _tiny("tiny_small", 1)
    toks = synth.make_prompt(16, cfg["vocab"], 9)
    one = _model(oracle_lib, cfg, ow).feed_block(toks, all_logits=True)
    m = _model(oracle_lib, cfg, ow)
    a = m.feed_block(toks[:split], all_logits=True)
    b = m.feed_block(toks[split:], all_logits=True)
    assert np.allclose(np.concatenate([a, b]), one, atol=1e-6)
    m = _model(oracle_lib, cfg, ow)
    m.feed_block(toks[:split])
    dec = np.stack([m.feed(toks[i:i + 1]) for i in range(split, 16)])
    assert np.allclose(dec, one[split:], atol=1e-6)
    want = bf.forward_all(cfg, ow, toks)
    assert np.abs(one - want).max() / np.abs(want).max() < 1e-5


def test_truncate_rolls_the_cache_back(oracle_lib):
    cfg, ow = _tiny("tiny_small", 1)
    toks = synth.make_prompt(12, cfg["vocab"], 10)
    m = _model(oracle_lib, cfg, ow)
    m.feed(toks[:8])
    m.feed(synth.make_prompt(4, cfg["vocab"], 11))          # a different continuation, then undone
    m.truncate(8)
    got = m.feed(toks[8:])
    want = _model(oracle_lib, cfg, ow).feed(toks)
    assert np.array_equal(got, want)
    with pytest.raises(ValueError):
        m.truncate(99)


def test_zero_output_projections_reduce_to_one_matvec(oracle_lib):
    """Wo = Wd = 0 => every layer is the identity on x => logits = W_lm rmsnorm(E[tok])."""
    cfg, ow = _tiny("tiny_small", 12)
    ow = dict(ow)
    ow["wo"] = [np.zeros_like(a) for a in ow["wo"]]
    ow["wd"] = [np.zeros_like(a) for a in ow["wd"]]
    toks = synth.make_prompt(5, cfg["vocab"], 13)
    got = _model(oracle_lib, cfg, ow).feed(toks)
    x = ow["embed"][toks[-1]].astype(np.float64)
    y = x / np.sqrt((x * x).mean() + cfg["rms_eps"]) * ow["final_norm"]
    want = ow["lm_head"].astype(np.float64) @ y
    assert np.allclose(got, want, atol=1e-6)


def test_zero_query_makes_attention_a_running_mean_of_values(oracle_lib):
    """Wq = bq = 0 and one layer with Wd = 0: x_out(p) = x_in(p) + Wo * mean_{j<=p} v_j."""
    cfg, ow = _tiny("tiny_small", 14, n_layers=1)
    ow = dict(ow)
    ow["wq"] = [np.zeros_like(ow["wq"][0])]
    ow["bq"] = [np.zeros_like(ow["bq"][0])]
    ow["wd"] = [np.zeros_like(ow["wd"][0])]
    for k in ("wk", "wv", "bk", "bv", "wo", "wg", "wu", "norm_attn", "norm_mlp"):
        ow[k] = ow[k][:1]
    toks = synth.make_prompt(6, cfg["vocab"], 15)
    got = _model(oracle_lib, cfg, ow).feed(toks)
    E = ow["embed"].astype(np.float64)
    X = E[toks]
    Y = X / np.sqrt((X * X).mean(axis=1, keepdims=True) + cfg["rms_eps"]) * ow["norm_attn"][0]
    Vv = Y @ ow["wv"][0].astype(np.float64).T + ow["bv"][0]                    # [T][nkv*d]
    vbar = Vv.mean(axis=0).reshape(cfg["n_kv_heads"], cfg["head_dim"])
    o = np.repeat(vbar, cfg["n_q_heads"] // cfg["n_kv_heads"], axis=0).reshape(-1)
    x = X[-1] + ow["wo"][0].astype(np.float64) @ o
    y = x / np.sqrt((x * x).mean() + cfg["rms_eps"]) * ow["final_norm"]
    want = ow["lm_head"].astype(np.float64) @ y
    assert np.allclose(got, want, atol=1e-6)


def test_feed_rejects_bad_input(oracle_lib):
    cfg, ow = _tiny("tiny_small", 1, max_seq=8)
    m = _model(oracle_lib, cfg, ow)
    with pytest.raises(ValueError):
        m.feed(np.array([cfg["vocab"]], np.int32))
    with pytest.raises(ValueError):
        m.feed(np.array([-1], np.int32))
    with pytest.raises(ValueError):
        m.feed(np.zeros(9, np.int32))
    m.feed(np.zeros(8, np.int32))
    with pytest.raises(ValueError):
        m.feed(np.zeros(1, np.int32))


def test_tied_head_uses_embedding(oracle_lib):
    cfg, ow = _tiny("tiny_small", 16)
    ow = dict(ow, lm_head=None)
    toks = synth.make_prompt(4, cfg["vocab"], 17)
    got = _model(oracle_lib, cfg, ow).feed(toks)
    want = bf.forward_all(cfg, ow, toks)[-1]
    assert np.abs(got - want).max() / np.abs(want).max() < 1e-5
