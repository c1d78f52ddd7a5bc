"""The decode step as one persistent kernel (ST_DECODE_PERSIST=1, st_decode_step_kind == 1) against the CPU oracle and
against the default kernel-per-stage step, through the C ABI: contexts that need one key range, several ranges and the range merge, ranges
of more than one tile, both head sizes, and the bounded wait."""
import os

import numpy as np
import pytest

from oracle import oracle as O
from paper_2504_12329_amd import binding as B, synth
from tests.gpu_common import LOGIT_TOL, make_pair, print_case, rel_err

pytestmark = pytest.mark.gpu


def _with_env(name, value, fn):
    old = os.environ.get(name)
    os.environ[name] = value
    try:
        return fn()
    finally:
        if old is None:
            del os.environ[name]
        else:
            os.environ[name] = old


def _persist_pair(*args, **kw):
    return _with_env("ST_DECODE_PERSIST", "1", lambda: make_pair(*args, **kw))


def test_tiny_model_both_step_kinds_against_the_oracle():
    """Teacher-forced decode from 20 to 215 keys (1 .. 4 ranges of 64 keys) on the tiny model: the single-kernel
    step and the kernel-per-stage step each within the logit tolerance of the oracle, same arg-max as their own
    logits, and within 1e-4 of each other."""
    cfg, g1, o = _persist_pair("tiny_small", 1, max_seq=256, max_chunk=64)
    _, g0, _ = make_pair("tiny_small", 1, max_seq=256, max_chunk=64)
    assert g1.step_kind() == 1 and g0.step_kind() == 0
    prompt = synth.make_prompt(20, cfg["vocab"], 5)
    print_case("tiny: 20-token prompt, 195 teacher-forced steps, both step kinds")
    tok = O.argmax(o.feed(prompt))
    g1.prefill(prompt, want_logits=False)
    g0.prefill(prompt, want_logits=False)
    worst1 = worst0 = apart = 0.0
    for step in range(195):
        lg_o = o.feed([tok])
        lg1, t1 = g1.decode_step(tok)
        lg0, t0 = g0.decode_step(tok)
        assert t1 == O.argmax(lg1) and t0 == O.argmax(lg0)
        worst1 = max(worst1, rel_err(lg1, lg_o))
        worst0 = max(worst0, rel_err(lg0, lg_o))
        apart = max(apart, rel_err(lg1, lg0))
        tok = O.argmax(lg_o)
    print_case("worst error: single kernel", worst1, "per stage", worst0, "apart", apart)
    assert worst1 <= LOGIT_TOL and worst0 <= LOGIT_TOL and apart <= 1e-4
    assert g1.kv_len == g0.kv_len == o.kv_len == 215
    # chained steps and the trigger predicate go through the same kernel
    a = g1.decode_greedy(tok, 12)
    b = g0.decode_greedy(tok, 12)
    assert a.tolist() == b.tolist()
    g1.close(), g0.close()


@pytest.mark.parametrize("name,layers,kv0", [("qwen1p5b", 2, 700), ("qwen7b", 2, 300), ("qwen32b", 1, 200)])
def test_paper_shapes_few_layers(name, layers, kv0):
    """The 1.5B / 7B / 32B shapes with a few layers: a prompt pass of kv0 tokens, then 6 teacher-forced single-kernel
    steps against the oracle (1.5B at 700 keys: eleven ranges and the merge; G = 6, 7, 5)."""
    cfg, g, o = _persist_pair(name, 3, max_seq=kv0 + 16, max_chunk=kv0, n_layers=layers, gen_device="cuda")
    assert g.step_kind() == 1
    prompt = synth.make_prompt(kv0, cfg["vocab"], 11)
    print_case(name, layers, "layers:", kv0, "prompt tokens, 6 single-kernel steps")
    tok = O.argmax(o.feed(prompt))
    g.prefill(prompt, want_logits=False)
    worst = 0.0
    for _ in range(6):
        lg_o = o.feed([tok])
        lg, t = g.decode_step(tok)
        assert t == O.argmax(lg)
        worst = max(worst, rel_err(lg, lg_o))
        tok = O.argmax(lg_o)
    print_case("worst error", worst)
    assert worst <= LOGIT_TOL
    g.close()


def test_long_ranges_take_several_tiles():
    """With 2 kv heads a context of 128 * 64 keys fills all ranges with one tile; beyond it ranges hold two tiles.
    A narrow model (hidden 256, head_dim 64) at 8300 keys: the single-kernel step equals the kernel-per-stage step to
    1e-4 and both match the oracle's logits at the last of 3 steps."""
    kv0 = 8300
    cfg, g1, o = _persist_pair("tiny_small", 7, max_seq=kv0 + 8, max_chunk=512)
    _, g0, _ = make_pair("tiny_small", 7, max_seq=kv0 + 8, max_chunk=512)
    assert g1.step_kind() == 1 and g0.step_kind() == 0
    prompt = synth.make_prompt(kv0, cfg["vocab"], 13)
    print_case("tiny at", kv0, "keys: two-tile ranges")
    g1.prefill(prompt, want_logits=False)
    g0.prefill(prompt, want_logits=False)
    tok = O.argmax(o.feed(prompt))
    for _ in range(3):
        lg_o = o.feed([tok])
        lg1, _ = g1.decode_step(tok)
        lg0, _ = g0.decode_step(tok)
        assert rel_err(lg1, lg0) <= 1e-4
        assert rel_err(lg1, lg_o) <= LOGIT_TOL
        tok = O.argmax(lg_o)
    g1.close(), g0.close()


def test_a_wait_that_runs_out_is_reported_and_truncate_recovers():
    """ST_PERSIST_SPIN=1 lets every wait inside the kernel give up after two polling rounds (the host forces the
    condition, every wave still exits normally): the step is reported as failed with ST_EHIP instead of returning
    wrong numbers silently, and st_kv_truncate clears the condition.  (Two rounds are not always too few on a model
    this small: the test accepts a step that succeeds, and then only checks its result.)"""
    cfg, g, o = _with_env("ST_PERSIST_SPIN", "1", lambda: _persist_pair("tiny_small", 1, max_seq=128, max_chunk=64))
    assert g.step_kind() == 1
    prompt = synth.make_prompt(40, cfg["vocab"], 5)
    tok = O.argmax(o.feed(prompt))
    g.prefill(prompt, want_logits=False)
    failed = 0
    for _ in range(8):
        try:
            lg, _ = g.decode_step(tok)
        except B.StError as e:
            assert e.code == B.ST_EHIP and "timed out" in str(e)
            failed += 1
            g.truncate(40)
            continue
        assert rel_err(lg, o.feed([tok])) <= LOGIT_TOL
        o.truncate(40)
        g.truncate(40)
    print_case("steps that gave up:", failed, "of 8")
    g.close()


def test_two_model_loop_on_the_single_kernel_step_matches_the_oracle_schedule():
    """The whole takeover loop (st_generate: speculative model, trigger rule, target segments, catch-up passes) with
    both tiny models on the single-kernel step: token sequence, sources and trigger positions equal the schedule
    oracle's (same prompt seed, margin-checked, as the kernel-per-stage test of the tiny pair)."""
    from oracle import schedule as S
    cfg, gs, os_ = _persist_pair("tiny_small", 1, max_seq=256, max_chunk=64)
    _, gl, ol = _persist_pair("tiny_large", 2, max_seq=256, max_chunk=64)
    assert gs.step_kind() == 1 and gl.step_kind() == 1
    prompt = synth.make_prompt(32, cfg["vocab"], 319)
    a, b = S.GreedyModel(os_, keep_logits=True), S.GreedyModel(ol, keep_logits=True)
    tr = S.speculative_thinking(a, b, prompt, 64, 8, S.window_rule(lambda t: t % 16 == 0))
    margin = min((np.sort(lg)[-1] - np.sort(lg)[-2]) / np.abs(lg).max() for g in (a, b) for _, lg in g.logits)
    assert margin >= 0.008 and len(tr.triggers) >= 2
    rule = B.TriggerRule(cfg["vocab"], synth.modulo_bitmap(cfg["vocab"], 16))
    print_case("tiny pair, single-kernel step: 64 outputs, segments of 8, triggers", tr.triggers)
    out = B.st_generate(gs, gl, rule, prompt, 64, 8)
    assert out["seq"].tolist() == tr.seq and out["src"].tolist() == tr.src
    assert [s["large_prefill_hi"] - 1 for s in out["spans"]] == tr.triggers
    gs.close(), gl.close()


def test_full_depth_1p5b_both_step_kinds_agree():
    """All 28 layers of the 1.5B shape at 600 .. 616 keys: the single-kernel step against the kernel-per-stage step
    (each pinned to the oracle elsewhere: the whole-model test of the default step, the few-layer test above), logits
    within 1e-3 of each other at every one of 16 chained steps' starting points and the same greedy tokens."""
    name, kv0 = "qwen1p5b", 600
    cfg = synth.model_config(name, max_seq=kv0 + 32, max_chunk=kv0)
    w = synth.make_weights(cfg, 4, device="cuda")
    g1 = _with_env("ST_DECODE_PERSIST", "1", lambda: B.Model(cfg, w))
    g0 = B.Model(cfg, w)
    assert g1.step_kind() == 1 and g0.step_kind() == 0
    prompt = synth.make_prompt(kv0, cfg["vocab"], 21)
    print_case("1.5B shape, 28 layers:", kv0, "prompt tokens, 16 steps on both step kinds")
    _, t1 = g1.prefill(prompt, want_logits=False)
    _, t0 = g0.prefill(prompt, want_logits=False)
    assert t1 == t0
    tok, apart = t0, 0.0
    for _ in range(16):
        lg1, n1 = g1.decode_step(tok)
        lg0, n0 = g0.decode_step(tok)
        apart = max(apart, rel_err(lg1, lg0))
        margin = (np.sort(lg0)[-1] - np.sort(lg0)[-2]) / np.abs(lg0).max()
        assert n1 == n0 or margin < 1e-3, (n1, n0, margin)
        tok = n0
    print_case("largest distance between the two step kinds", apart)
    assert apart <= 1e-3
    g1.close(), g0.close()


@pytest.mark.parametrize("d,nq,nkv", [(64, 4, 4), (128, 3, 1), (64, 8, 2), (128, 8, 1), (128, 16, 16)])
def test_every_head_grouping_on_both_step_kinds(d, nq, nkv):
    """Query heads per kv head G = 1, 3, 4, 8 (and 16 kv heads of one query head each) at both head sizes, on a narrow
    two-layer model (hidden 512, intermediate 1032 -- rows of 129 sixteen-byte groups, not a multiple of a wave --
    vocabulary 2000): 70-token prompt, then 6 teacher-forced steps across the 64-key range boundary, both step kinds
    against the oracle."""
    over = dict(head_dim=d, n_q_heads=nq, n_kv_heads=nkv, hidden=512, intermediate=1032, vocab=2000)
    cfg, g1, o = _persist_pair("tiny_small", 9, max_seq=128, max_chunk=80, **over)
    _, g0, _ = make_pair("tiny_small", 9, max_seq=128, max_chunk=80, **over)
    assert g1.step_kind() == 1 and g0.step_kind() == 0
    prompt = synth.make_prompt(60, cfg["vocab"], 17)
    print_case("head_dim", d, "q heads", nq, "kv heads", nkv, ": 60-token prompt, 8 steps")
    tok = O.argmax(o.feed(prompt))
    g1.prefill(prompt, want_logits=False)
    g0.prefill(prompt, want_logits=False)
    for _ in range(8):
        lg_o = o.feed([tok])
        lg1, t1 = g1.decode_step(tok)
        lg0, t0 = g0.decode_step(tok)
        assert t1 == O.argmax(lg1) and t0 == O.argmax(lg0)
        assert rel_err(lg1, lg_o) <= LOGIT_TOL and rel_err(lg0, lg_o) <= LOGIT_TOL and rel_err(lg1, lg0) <= 1e-4
        tok = O.argmax(lg_o)
    g1.close(), g0.close()
