"""Trigger-scan oracle against a brute-force loop, and the work counters against Appendix A."""
import numpy as np
import pytest

from paper_2504_12329_amd import cost, synth


def _brute(tokens, lo, hi, kwset, delimset, window):
    """Window 1: keyword positions.  Otherwise the sentence bookkeeping of the takeover policy replayed from the
    first token: a delimiter arms the sentence that starts after it (a delimiter inside re-arms it); the position
    where a sentence of window - 1 tokens completes fires when the sentence holds a keyword."""
    if window == 1:
        return [p for p in range(lo, hi) if tokens[p] in kwset]
    w, start, out = window - 1, None, []
    for q in range(len(tokens)):
        if start is not None and q == start + w - 1:
            if lo <= q < hi and any(t in kwset for t in tokens[start:q + 1]):
                out.append(q)
            start = None
        if tokens[q] in delimset:
            start = q + 1
    return out


def test_modulo_bitmap():
    bm = synth.modulo_bitmap(1024, 16)
    ids = [i for i in range(1024) if (bm[i >> 5] >> (i & 31)) & 1]
    assert ids == list(range(0, 1024, 16))
    bm = synth.modulo_bitmap(151936, 97)
    assert sum(bin(int(x)).count("1") for x in bm) == len(range(0, 151936, 97))


@pytest.mark.parametrize("window", [1, 2, 3, 5, 21])
def test_trigger_scan_bruteforce(oracle_lib, window):
    rng = np.random.default_rng(window)
    V = 300
    kw, dl = synth.modulo_bitmap(V, 7), synth.modulo_bitmap(V, 3)
    kwset, dlset = set(range(0, V, 7)), set(range(0, V, 3))
    for trial in range(30):
        n = int(rng.integers(0, 200))
        toks = rng.integers(0, V, n).astype(np.int32)
        if window > 2 and n:                  # long windows need sparse delimiters to fire at all
            toks[toks % 3 == 0] += 1
            toks[rng.integers(0, n, max(1, n // (2 * window)))] = 3 * rng.integers(0, V // 3, max(1, n // (2 * window)))
        if n > 3:
            toks[0] = 0                       # id 0 is divisible by everything; p = 0 has no predecessor
            toks[rng.integers(0, n)] = 21
        lo = int(rng.integers(0, n + 1))
        hi = int(rng.integers(lo, n + 1))
        want = _brute(toks, lo, hi, kwset, dlset, window)
        cnt, pos = oracle_lib.trigger_scan(toks, lo, hi, V, kw, dl, window, cap=1000)
        assert cnt == len(want) and pos.tolist() == want
        cnt, pos = oracle_lib.trigger_scan(toks, lo, hi, V, kw, dl, window, cap=2)
        assert cnt == len(want) and pos.tolist() == want[:2]


def _running_maxima(tokens, lo, hi, kwset, delimset, window):
    """The form the GPU scan evaluates (host arithmetic of k_trigger_scan): with w = window - 1, lastD(q) / lastK(q)
    the largest index <= q holding a delimiter / keyword, p fires when p - w >= 0, lastD(p - 1) == p - w and
    lastK(p) > p - w; the running maxima start w tokens before lo."""
    if window == 1:
        return [p for p in range(lo, hi) if tokens[p] in kwset]
    w, out = window - 1, []
    last_d = last_k = -1
    for p in range(max(0, lo - w), hi):
        before_d = last_d
        if tokens[p] in delimset:
            last_d = p
        if tokens[p] in kwset:
            last_k = p
        if p >= lo and p - w >= 0 and before_d == p - w and last_k > p - w:
            out.append(p)
    return out


@pytest.mark.parametrize("window", [2, 3, 4, 9, 40, 257])
def test_running_maxima_form_of_the_rule(oracle_lib, window):
    """The prefix-scan form of the sentence rule gives the positions of the brute-force replay and of the oracle."""
    rng = np.random.default_rng(100 + window)
    V = 120
    kw, dl = synth.modulo_bitmap(V, 7), synth.modulo_bitmap(V, 3)
    kwset, dlset = set(range(0, V, 7)), set(range(0, V, 3))
    for trial in range(40):
        n = int(rng.integers(0, 700))
        toks = rng.integers(0, V, n).astype(np.int32)
        if n:                                 # delimiters about one sentence apart, so that long windows fire too
            toks[toks % 3 == 0] += 1
            k = max(1, n // window)
            toks[rng.integers(0, n, k)] = 3 * rng.integers(0, V // 3, k)
        lo = int(rng.integers(0, n + 1))
        hi = int(rng.integers(lo, n + 1))
        got = _running_maxima(toks, lo, hi, kwset, dlset, window)
        assert got == _brute(toks, lo, hi, kwset, dlset, window)
        assert got == oracle_lib.trigger_scan(toks, lo, hi, V, kw, dl, window, cap=1000)[1].tolist()


def test_trigger_scan_hand_cases(oracle_lib):
    V = 64
    kw, dl = synth.modulo_bitmap(V, 5), synth.modulo_bitmap(V, 3)
    toks = np.array([5, 3, 5, 10, 9, 4, 15, 6, 20], np.int32)
    assert oracle_lib.trigger_scan(toks, 0, 9, V, kw, dl, 2, 9)[1].tolist() == [2, 8]
    assert oracle_lib.trigger_scan(toks, 0, 9, V, kw, dl, 1, 9)[1].tolist() == [0, 2, 3, 6, 8]
    assert oracle_lib.trigger_scan(toks, 2, 3, V, kw, dl, 2, 9)[1].tolist() == [2]   # looks back before lo
    assert oracle_lib.trigger_scan(toks, 4, 4, V, kw, dl, 1, 9)[0] == 0              # empty range
    # sentences of 3 tokens (window 4) worked by hand; ids: delimiter % 3, keyword % 5
    #        pos 0  1  2  3  4  5   6  7  8  9  10 11 12 13 14
    toks = np.array([1, 3, 7, 8, 5, 2, 6, 4, 9, 10, 7, 3, 1, 1, 20], np.int32)
    # 3@1 arms (2,3,4): 5 at 4 -> fires at 4.  6@6 arms (7,8,9) but 9@8 is a delimiter inside -> re-armed at 9:
    # (9,10,11) holds 10 and ends on a delimiter (allowed) -> fires at 11.  3@11 arms (12,13,14): 20 -> fires at 14.
    assert oracle_lib.trigger_scan(toks, 0, 15, V, kw, dl, 4, 9)[1].tolist() == [4, 11, 14]
    assert oracle_lib.trigger_scan(toks, 5, 14, V, kw, dl, 4, 9)[1].tolist() == [11]
    with pytest.raises(ValueError):
        oracle_lib.trigger_scan(np.array([64], np.int32), 0, 1, V, kw, dl, 1, 4)


def test_cost_reduces_to_appendix_a_for_mha():
    # Appendix A, per layer, h = n*d:  decode(s) = 8h^2 + 16h + 4sh + 4sn + 6hh' + 2h'
    #                                  prefill(s) = 8sh^2 + 16sh + 4s^2h + 4s^2n + 6shh' + 2sh'
    # the 16h, 4sn, 2h' terms are element-wise work; the counter keeps the matmul terms.
    n, d, hp = 12, 128, 8960
    h = n * d
    cfg = dict(hidden=h, head_dim=d, n_q_heads=n, n_kv_heads=n, intermediate=hp, n_layers=1, vocab=1000)
    for s in (1, 17, 4096):
        assert cost.decode_flops_layer(cfg, s) == 8 * h * h + 4 * s * h + 6 * h * hp
        assert cost.prefill_flops_layer(cfg, s, 0, causal=False) == 8 * s * h * h + 4 * s * s * h + 6 * s * h * hp
    # a prefix pass of m tokens on a cache of kv0 costs what m decode steps at growing lengths cost
    m, kv0 = 9, 100
    assert cost.prefill_flops_layer(cfg, m, kv0) == sum(cost.decode_flops_layer(cfg, kv0 + i + 1) for i in range(m))


def test_cost_bytes_of_the_paper_models():
    c15 = synth.model_config("qwen1p5b", 4608)
    c32 = synth.model_config("qwen32b", 8192)
    assert cost.layer_matmul_params(c15) == 46792704
    assert cost.layer_matmul_params(c32) == 487587840
    assert abs(cost.weight_bytes(c15) / 1e9 - 3.087) < 1e-3
    assert abs(cost.weight_bytes(c32) / 1e9 - 63.97) < 1e-2
    assert cost.kv_bytes_per_position(c15) == 28672 and cost.kv_bytes_per_position(c32) == 262144
