"""The takeover schedule oracle against a trace worked by hand (stub models), and its edge cases."""
import os

import pytest

from oracle import schedule as S

GOLD = os.path.join(os.path.dirname(__file__), "golden", "schedule_hand_trace.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        out[k] = v
    spans = lambda k: [tuple(int(x) for x in s.split(":")) for s in out[k]]
    return dict(prompt=[int(x) for x in out["prompt"]], n_out=int(out["n_out"][0]), n_seg=int(out["n_seg"][0]),
                triggers=[int(x) for x in out["triggers"]], large_prefill=spans("large_prefill"),
                large_decode=spans("large_decode"), small_prefill=spans("small_prefill"),
                feeds=int(out["large_decode_feeds"][0]), src=out["src"][0], seq=[int(x) for x in out["seq"]],
                ratio=out["modify_ratio"][0])


class Stub:
    """Emits f(position being written); checks that it is fed exactly the tokens it has not seen."""

    def __init__(self, f, seq_ref):
        self.f, self.kv, self.seq_ref, self.fed = f, 0, seq_ref, []

    def feed(self, tokens):
        tokens = list(tokens)
        assert len(tokens) >= 1
        self.fed.append((self.kv, self.kv + len(tokens)))
        self.kv += len(tokens)
        return self.f(self.kv)


def test_hand_trace():
    g = _gold()
    small = Stub(lambda p: p, None)
    large = Stub(lambda p: 495 + p, None)
    fire = S.window_rule(lambda t: t % 16 == 0)
    tr = S.speculative_thinking(small, large, g["prompt"], g["n_out"], g["n_seg"], fire)
    assert tr.seq == g["seq"]
    assert tr.triggers == g["triggers"]
    assert tr.large_prefill == g["large_prefill"]
    assert tr.large_decode == g["large_decode"]
    assert tr.small_prefill == g["small_prefill"]
    assert tr.large_decode_feeds == g["feeds"]
    assert "".join("SL"[s] for s in tr.src) == g["src"]
    num, den = (int(x) for x in g["ratio"].split("/"))
    assert abs(tr.modify_ratio - num / den) < 1e-12
    # every model saw a gap-free, overlap-free token stream
    for m in (small, large):
        for (a, b), (c, d) in zip(m.fed, m.fed[1:]):
            assert b == c


def test_budget_ends_on_trigger_token_means_no_handoff():
    small = Stub(lambda p: p, None)
    large = Stub(lambda p: 495 + p, None)
    fire = S.window_rule(lambda t: t % 16 == 0)
    tr = S.speculative_thinking(small, large, [1, 2, 3, 5], 13, 8, fire)        # 13th output is id 16
    assert tr.seq[-1] == 16 and tr.triggers == [] and tr.large_prefill == [] and len(tr.src) == 13
    assert large.fed == [(0, 4)]                                               # only the prompt


def test_window_two_needs_delimiter_before_keyword():
    kw = lambda t: t % 5 == 0
    delim = lambda t: t % 3 == 0
    fire = S.window_rule(kw, delim, window=2)
    seq = [5, 3, 5, 10, 9, 4, 15, 6, 20]
    assert [p for p in range(len(seq)) if fire(seq, p)] == [2, 8]
    assert not fire([5], 0)                                                   # no previous token at p = 0
    # the previous token may be the last prompt token
    small = Stub(lambda p: 5 * p, None)
    large = Stub(lambda p: 1000 + p, None)
    tr = S.speculative_thinking(small, large, [7, 9], 6, 2, fire)
    assert tr.triggers == [2]                                                 # seq[1] = 9 (delim), seq[2] = 10 (kw)
    assert tr.seq == [7, 9, 10, 1003, 1004, 25, 30, 35]
    assert tr.small_prefill == [(2, 5)] and tr.large_prefill == [(2, 3)]


def test_zero_budget_and_full_segment_at_budget():
    small = Stub(lambda p: 16, None)          # every small token triggers
    large = Stub(lambda p: 1, None)
    fire = S.window_rule(lambda t: t % 16 == 0)
    assert S.speculative_thinking(small, large, [3], 0, 4, fire).seq == [3]
    tr = S.speculative_thinking(small, large, [3], 5, 4, fire)                 # S LLLL -> exactly the budget
    assert "".join("SL"[s] for s in tr.src) == "SLLLL" and tr.small_prefill == []
    tr = S.speculative_thinking(small, large, [3], 7, 4, fire)                 # S LLLL S L
    assert "".join("SL"[s] for s in tr.src) == "SLLLLSL"
    assert tr.small_prefill == [(1, 6)] and tr.large_prefill == [(1, 2), (5, 7)]


def test_paper_hyperparameters_fixture():
    vals = dict(l.split() for l in open(os.path.join(os.path.dirname(GOLD), "paper_hyperparameters.txt"))
                if l.strip() and not l.startswith("#"))
    from paper_2504_12329_amd import defaults
    assert defaults.N1 == int(vals["n1"]) and defaults.N2 == int(vals["n2"]) and defaults.N3 == int(vals["n3"])
    assert defaults.REFLECTION_THRESHOLD == int(vals["reflection_threshold"])
    assert defaults.INITIAL_TARGET_TOKENS == int(vals["initial_target_tokens"])
