"""GPU parity of the whole path on the tiny model pair against the CPU oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

from oracle import oracle as O, schedule as S
from paper_2504_12329_amd import binding as B, synth
from tests.gpu_common import LOGIT_TOL, make_pair, print_case, rel_err

pytestmark = pytest.mark.gpu

# Greedy decoding of random-init weights has near-ties; a bf16 path may then legitimately pick the
# other token.  The prompt seeds below were searched on the CPU so that, in the oracle's own run of
# each scenario, every top-1/top-2 logit gap is at least MIN_MARGIN of max|logit| (3x the worst GPU
# logit error seen on these models); each test re-checks that margin before comparing tokens.
PROMPT_SEED = 319            # mod-16 rule, 64 outputs, segments of 8
PROMPT_SEED_WINDOW2 = 477    # (prev % 3 == 0 and tok % 2 == 0) rule, segments of 5
PROMPT_SEED_FORCED = 293     # hand-over every 6th speculative token, segments of 4
PROMPT_SEED_GREEDY = 26      # the small model alone, 44 greedy steps
MIN_MARGIN = 0.008
N_OUT, N_SEG = 64, 8


@pytest.fixture(scope="module")
def small():
    cfg, g, o = make_pair("tiny_small", 1, max_seq=256, max_chunk=64)
    yield cfg, g, o
    g.close()


def _fresh(g, o):
    g.truncate(0)
    o.truncate(0)


def test_prefill_and_teacher_forced_decode_logits(small):
    cfg, g, o = small
    _fresh(g, o)
    prompt = synth.make_prompt(32, cfg["vocab"], 3)
    print_case("tiny prefill 32 + 64 teacher-forced decode steps")
    lg_o = o.feed(prompt)
    lg_g, tok_g = g.prefill(prompt)
    assert rel_err(lg_g, lg_o) <= LOGIT_TOL
    assert tok_g == O.argmax(lg_g)                        # the kernel's arg-max of its own logits
    worst = 0.0
    tok = O.argmax(lg_o)
    for step in range(64):
        lg_o = o.feed([tok])
        lg_g, tok_g = g.decode_step(tok)
        worst = max(worst, rel_err(lg_g, lg_o))
        assert tok_g == O.argmax(lg_g)
        tok = O.argmax(lg_o)                              # teacher forcing: both sides follow the oracle
    print_case("worst relative logit error", worst)
    assert worst <= LOGIT_TOL
    assert g.kv_len == o.kv_len == 96


def test_greedy_tokens_identical(small):
    cfg, g, o = small
    _fresh(g, o)
    prompt = synth.make_prompt(32, cfg["vocab"], PROMPT_SEED_GREEDY)
    tok_o = O.argmax(o.feed(prompt))
    _, tok_g = g.prefill(prompt, want_logits=False)
    assert tok_g == tok_o
    want = []
    t = tok_o
    margins = []
    for _ in range(44):
        lg = o.feed([t])
        t = O.argmax(lg)
        want.append(t)
        margins.append((np.sort(lg)[-1] - np.sort(lg)[-2]) / np.abs(lg).max())
    assert min(margins) >= MIN_MARGIN, f"near-tie in the oracle run: {min(margins):.4f}"
    got = g.decode_greedy(tok_g, 40)
    print_case("greedy", got[:40].tolist())
    assert got.tolist() == want[:40]
    # chained continuation picks up the device-resident token
    more = g.decode_greedy(0, 4, chained=True)
    assert more.tolist() == want[40:]


@pytest.mark.parametrize("split", [1, 7, 31, 45])
def test_chunked_prefill(small, split):
    cfg, g, o = small
    prompt = synth.make_prompt(70, cfg["vocab"], 5)       # 70 > max_chunk 64: the library splits internally too
    _fresh(g, o)
    want = o.feed(prompt)
    g.prefill(prompt[:split], want_logits=False)
    got, _ = g.prefill(prompt[split:])
    assert rel_err(got, want) <= LOGIT_TOL
    _fresh(g, o)
    one, _ = g.prefill(prompt)
    assert rel_err(one, want) <= LOGIT_TOL
    assert g.kv_len == 70


def test_truncate_and_determinism(small):
    cfg, g, o = small
    prompt = synth.make_prompt(40, cfg["vocab"], 6)
    runs = []
    for _ in range(3):
        g.truncate(0)
        g.prefill(prompt[:30], want_logits=False)
        g.prefill(synth.make_prompt(10, cfg["vocab"], 7), want_logits=False)   # wrong continuation, rolled back
        g.truncate(30)
        lg, _ = g.prefill(prompt[30:])
        for t in (1, 2, 3):
            lg2, _ = g.decode_step(t)
        runs.append((lg.copy(), lg2.copy()))
    for a, b in runs[1:]:
        assert np.array_equal(a, runs[0][0]) and np.array_equal(b, runs[0][1])   # bit-identical across runs
    o.truncate(0)
    assert rel_err(runs[0][0], o.feed(prompt)) <= LOGIT_TOL


def test_error_paths_on_device(small):
    cfg, g, o = small
    g.truncate(0)
    with pytest.raises(B.StError) as e:
        g.prefill(np.zeros(257, np.int32))
    assert e.value.code == B.ST_ERANGE and g.kv_len == 0
    with pytest.raises(B.StError) as e:
        g.prefill(np.array([5, cfg["vocab"]], np.int32))
    assert e.value.code == B.ST_ERANGE and g.kv_len == 0
    with pytest.raises(B.StError):
        g.prefill(np.zeros(0, np.int32))
    g.prefill(np.zeros(256, np.int32), want_logits=False)
    with pytest.raises(B.StError) as e:
        g.decode_step(1)
    assert e.value.code == B.ST_ERANGE and g.kv_len == 256
    with pytest.raises(B.StError):
        g.truncate(300)
    g.truncate(0)
    with pytest.raises(B.StError):
        g.decode_step(-1)
    with pytest.raises(B.StError):
        g.decode_greedy(0, 0)


def _oracle_trace(prompt, n_out, n_seg, fire, o_small, o_large):
    o_small.truncate(0)
    o_large.truncate(0)
    a, b = S.GreedyModel(o_small, keep_logits=True), S.GreedyModel(o_large, keep_logits=True)
    tr = S.speculative_thinking(a, b, prompt, n_out, n_seg, fire)
    margin = min((np.sort(lg)[-1] - np.sort(lg)[-2]) / np.abs(lg).max() for g in (a, b) for _, lg in g.logits)
    assert margin >= MIN_MARGIN, f"oracle run has a near-tie (margin {margin:.4f}); pick another prompt seed"
    return tr


@pytest.fixture(scope="module")
def pair(small):
    cfg_l, g_l, o_l = make_pair("tiny_large", 2, max_seq=256, max_chunk=64)
    yield small, (cfg_l, g_l, o_l)
    g_l.close()


def test_generate_matches_oracle_schedule(pair):
    (cfg, gs, os_), (_, gl, ol) = pair
    prompt = synth.make_prompt(32, cfg["vocab"], PROMPT_SEED)
    tr = _oracle_trace(prompt, N_OUT, N_SEG, S.window_rule(lambda t: t % 16 == 0), os_, ol)
    assert len(tr.triggers) >= 2
    gs.truncate(0)
    gl.truncate(0)
    rule = B.TriggerRule(cfg["vocab"], synth.modulo_bitmap(cfg["vocab"], 16))
    out = B.st_generate(gs, gl, rule, prompt, N_OUT, N_SEG)
    print_case("oracle triggers", tr.triggers, "gpu handoffs", out["stats"]["n_handoffs"])
    assert out["seq"].tolist() == tr.seq
    assert out["src"].tolist() == tr.src
    assert [(s["large_prefill_lo"], s["large_prefill_hi"]) for s in out["spans"]] == tr.large_prefill
    assert [(s["large_decode_lo"], s["large_decode_hi"]) for s in out["spans"]] == tr.large_decode
    assert [(s["small_prefill_lo"], s["small_prefill_hi"]) for s in out["spans"]
            if s["small_prefill_hi"] > s["small_prefill_lo"]] == tr.small_prefill
    assert [s["large_prefill_hi"] - 1 for s in out["spans"]] == tr.triggers
    assert out["stats"]["n_large"] == sum(tr.src) and out["stats"]["n_out"] == N_OUT
    # the scan kernel over the finished sequence finds the same trigger positions among small-written tokens
    seq_dev = torch.from_numpy(out["seq"]).cuda()
    cnt, pos = B.st_trigger_scan(rule, seq_dev, 32, 32 + N_OUT, cap=64)
    small_written = [p for p in pos.tolist() if out["src"][p - 32] == 0 and p < 32 + N_OUT - 1]
    assert small_written == tr.triggers


def test_generate_window_two_and_budget_inside_segment(pair):
    (cfg, gs, os_), (_, gl, ol) = pair
    prompt = synth.make_prompt(32, cfg["vocab"], PROMPT_SEED_WINDOW2)
    kw, dl = (lambda t: t % 2 == 0), (lambda t: t % 3 == 0)
    for n_out in (57, 29):                               # 29 outputs end inside the third segment
        tr = _oracle_trace(prompt, n_out, 5, S.window_rule(kw, dl, 2), os_, ol)
        gs.truncate(0)
        gl.truncate(0)
        rule = B.TriggerRule(cfg["vocab"], synth.modulo_bitmap(cfg["vocab"], 2), synth.modulo_bitmap(cfg["vocab"], 3), 2)
        out = B.st_generate(gs, gl, rule, prompt, n_out, 5)
        print_case("window-2 run", n_out, "triggers", tr.triggers)
        assert out["seq"].tolist() == tr.seq and out["src"].tolist() == tr.src
        assert [s["large_prefill_hi"] - 1 for s in out["spans"]] == tr.triggers
        if n_out == 29:
            assert tr.src[-1] == S.LARGE and len(tr.small_prefill) == len(tr.triggers) - 1


def test_forced_period_schedule(pair):
    (cfg, gs, os_), (_, gl, ol) = pair
    prompt = synth.make_prompt(32, cfg["vocab"], PROMPT_SEED_FORCED)
    count = {"n": 0}

    def fire(seq, p):                                   # every 6th small-written token hands over
        count["n"] += 1
        return count["n"] % 6 == 0
    tr = _oracle_trace(prompt, 50, 4, fire, os_, ol)
    gs.truncate(0)
    gl.truncate(0)
    out = B.st_generate(gs, gl, None, prompt, 50, 4, forced_period=6)
    assert out["seq"].tolist() == tr.seq and out["src"].tolist() == tr.src
    assert out["stats"]["n_handoffs"] == len(tr.triggers)


def test_single_handoff_call(pair):
    (cfg, gs, os_), (_, gl, ol) = pair
    prompt = synth.make_prompt(32, cfg["vocab"], PROMPT_SEED)
    for m in (gs, gl, os_, ol):
        m.truncate(0)
    seq = np.zeros(128, np.int32)
    seq[:32] = prompt
    _, tok = gs.prefill(prompt, want_logits=False)
    gl.prefill(prompt, want_logits=False)
    t_o = O.argmax(os_.feed(prompt))
    ol.feed(prompt)
    assert tok == t_o
    T = 32
    for _ in range(5):                                   # five small tokens, the last one is "the trigger"
        seq[T] = tok
        T += 1
        if T < 37:
            _, tok = gs.decode_step(tok, want_logits=False)
            assert tok == O.argmax(os_.feed([seq[T - 1]]))
    newT, nxt, sp, lg = B.st_handoff(gs, gl, seq, T, 8, 100, want_logits=True)
    # oracle: large catches up on [32,37), writes 8, is fed 7; small catches up on [36,45)
    tl = O.argmax(ol.feed(seq[32:37]))
    want = []
    for j in range(8):
        want.append(tl)
        if j < 7:
            tl = O.argmax(ol.feed([tl]))
    assert newT == 45 and seq[37:45].tolist() == want
    lo = os_.feed(np.concatenate([seq[36:37], np.array(want, np.int32)]))
    assert rel_err(lg, lo) <= LOGIT_TOL and nxt == O.argmax(lo)
    assert sp == dict(large_prefill_lo=32, large_prefill_hi=37, large_decode_lo=37, large_decode_hi=45,
                      small_prefill_lo=36, small_prefill_hi=45)
    assert gs.kv_len == 45 and gl.kv_len == 44
    with pytest.raises(B.StError):                       # both models already hold the whole sequence prefix
        B.st_handoff(gs, gl, seq, 44, 8, 100)


@pytest.mark.parametrize("window", [1, 2, 4, 21])
def test_trigger_scan_bit_exact(window):
    rng = np.random.default_rng(10 + window)
    V = 151936
    kw, dl = synth.modulo_bitmap(V, 97), synth.modulo_bitmap(V, 89)
    rule = B.TriggerRule(V, kw, dl, window)
    for n, lo, hi in [(0, 0, 0), (1, 0, 1), (1000, 0, 1000), (1024, 0, 1024), (1025, 1, 1025), (6000, 17, 5999),
                      (20000, 0, 20000), (3000, 2999, 3000), (3000, 1500, 1500)]:
        toks = rng.integers(0, V, max(n, 1)).astype(np.int32)
        if n > 10:                                       # plant hits, id 0, adjacent pairs, range borders
            idx = rng.integers(1, n, 40)
            toks[idx] = 97 * rng.integers(0, 1500, 40)
            toks[idx - 1] = 89 * rng.integers(0, 1700, 40)
            back = np.maximum(idx - rng.integers(1, max(window, 2), 40), 0)   # delimiters up to a sentence back
            toks[back] = 89 * rng.integers(0, 1700, 40)
            toks[0] = 0
            toks[n - 1] = 97
            toks[n - 2] = 89
        want_n, want_pos = O.trigger_scan(toks, lo, hi, V, kw, dl, window, cap=50)
        got_n, got_pos = B.st_trigger_scan(rule, torch.from_numpy(toks).cuda(), lo, hi, cap=50)
        assert got_n == want_n and got_pos.tolist() == want_pos.tolist(), (n, lo, hi)
        got_n, got_pos = B.st_trigger_scan(rule, torch.from_numpy(toks).cuda(), lo, hi, cap=3)
        assert got_n == want_n and got_pos.tolist() == want_pos.tolist()[:3]
    with pytest.raises(B.StError):
        B.st_trigger_scan(B.TriggerRule(V, kw, dl, 300), torch.zeros(4, dtype=torch.int32).cuda(), 0, 4, cap=4)
    # ids outside the vocabulary never fire on the device (the oracle rejects them outright)
    small_rule = B.TriggerRule(64, synth.modulo_bitmap(64, 1))
    toks = np.array([3, 64, -1, 5, 1 << 30], np.int32)
    n_, pos = B.st_trigger_scan(small_rule, torch.from_numpy(toks).cuda(), 0, 5, cap=8)
    assert n_ == 2 and pos.tolist() == [0, 3]


def test_decode_steps_replay_captured_graphs():
    """st_decode_graph_state: after a few decode steps the model reports captured step graphs in use (mode 0); with one
    kernel per stage the count grows when the context crosses into the next attention-grid bucket, the single-kernel
    step needs one graph for every length."""
    cfg = synth.model_config("tiny_small", max_seq=256, max_chunk=64)
    w = synth.make_weights(cfg, 1)
    wg = dict(embed=w["embed"].cuda(), final_norm=w["final_norm"].cuda(), lm_head=w["lm_head"].cuda(),
              layers=[{k: v.cuda() for k, v in lw.items()} for lw in w["layers"]])
    g = B.Model(cfg, wg)
    assert g.graph_state() == (0, 0)
    g.prefill(synth.make_prompt(60, cfg["vocab"], 3), want_logits=False)
    for t in range(3):
        g.decode_step(t + 1, want_logits=False)            # 61..63 keys: one range
    n1, mode = g.graph_state()
    assert mode == 0 and n1 >= 1
    for t in range(4):
        g.decode_step(t + 5, want_logits=False)            # 64..67 keys: two ranges, another graph
    n2, mode = g.graph_state()
    assert mode == 0 and (n2 == n1 if g.step_kind() == 1 else n2 > n1)
    g.close()
