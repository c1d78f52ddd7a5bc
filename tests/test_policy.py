"""The full-policy schedule oracle (Section 3 (1)-(3), replace reading, non-reasoning schedule) against traces
worked by hand with stub models, and its invariants."""
import os

import pytest

from oracle import schedule as S

GOLD = os.path.join(os.path.dirname(__file__), "golden", "policy_hand_traces.txt")


def gold_scenarios():
    out, cur = {}, None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        if k == "scenario":
            cur = out.setdefault(v[0], {})
        else:
            cur[k] = v
    return out


def spans(v):
    return [tuple(int(x) for x in s.split(":")) for s in v]


class Stub:
    """Emits base + (position being written); checks that it is fed exactly the tokens it has not seen."""

    def __init__(self, base):
        self.base, self.kv, self.fed = base, 0, []

    def feed(self, tokens):
        tokens = list(tokens)
        assert len(tokens) >= 1
        self.fed.append((self.kv, self.kv + len(tokens)))
        self.kv += len(tokens)
        return self.base + self.kv

    def truncate(self, n):
        assert 0 <= n <= self.kv
        self.kv = n


POLICIES = {
    "R": (500, S.Policy(delim=lambda t: t % 6 == 0, sentence_len=3, ar=lambda t: t % 10 == 0, n1=3, replace=True)),
    "V": (700, S.Policy(delim=lambda t: t % 7 == 0, sentence_len=2, verify=lambda t: t % 5 == 0, n2=16)),
    "E": (500, S.Policy(delim=lambda t: t % 6 == 0, sentence_len=2, neg=lambda t: t % 4 == 0, neg_threshold=1,
                        aux=(901, 902), n3=3)),
    "N": (500, S.Policy(delim=lambda t: t % 6 == 0, sentence_len=1, unconditional=True, n1=2, initial_target=5)),
}


@pytest.mark.parametrize("name", sorted(POLICIES))
def test_policy_hand_trace(name):
    g = gold_scenarios()[name]
    base, pol = POLICIES[name]
    small, large = Stub(0), Stub(base)
    prompt = [int(x) for x in g["prompt"]]
    tr = S.speculative_thinking_policy(small, large, prompt, int(g["n_out"][0]), pol)
    assert tr.seq == [int(x) for x in g["seq"]]
    assert "".join("SLA"[s] for s in tr.src) == g["src"][0]
    assert tr.actions == spans(g["actions"])
    assert tr.small_feeds == spans(g["small_feeds"]) and tr.large_feeds == spans(g["large_feeds"])
    assert tr.small_truncates == [int(x) for x in g.get("small_truncates", [])]
    assert tr.large_truncates == [int(x) for x in g.get("large_truncates", [])]
    assert len(tr.src) == int(g["n_out"][0]) == len(tr.seq) - len(prompt)


def test_policy_reduces_to_the_single_keyword_rule():
    """sentence_len 1, append, only (1): the same sequence and hand-over points as the window-2 rule."""
    kw, delim = (lambda t: t % 5 == 0), (lambda t: t % 3 == 0)
    a = S.speculative_thinking(Stub(0), Stub(495), [1, 2, 4, 7], 40, 4, S.window_rule(kw, delim, window=2))
    b = S.speculative_thinking_policy(Stub(0), Stub(495), [1, 2, 4, 7], 40,
                                      S.Policy(delim=delim, sentence_len=1, ar=kw, n1=4))
    assert a.seq == b.seq and a.src == b.src
    assert a.triggers == [act[1] for act in b.actions]


def test_each_model_is_fed_every_kept_token_once_and_in_order():
    for name, (base, pol) in POLICIES.items():
        small, large = Stub(0), Stub(base)
        tr = S.speculative_thinking_policy(small, large, [1, 2, 3, 5], 200, pol)
        for feeds, cuts in ((tr.small_feeds, tr.small_truncates), (tr.large_feeds, tr.large_truncates)):
            kv = 0
            cuts = list(cuts)
            for lo, hi in feeds:
                if lo != kv:                       # only a truncation may move the cursor back
                    assert cuts and cuts.pop(0) == lo and lo < kv
                assert hi > lo
                kv = hi
            assert kv <= len(tr.seq)
        assert len(tr.src) == 200


def test_budget_spent_inside_the_auxiliary_sentence():
    base, pol = POLICIES["E"]
    tr = S.speculative_thinking_policy(Stub(0), Stub(base), [1, 2, 3, 5], 18, pol)   # 17 small tokens + 1 of 2 aux
    assert tr.seq[-1] == 901 and tr.src[-1] == S.AUX and len(tr.src) == 18
    assert tr.large_feeds == [(0, 4)]


def test_replaced_sentence_right_after_the_prompt():
    """The prompt ends on a delimiter and the first sentence is replaced: the target has nothing to catch up on
    and writes from its prediction after the prompt."""
    pol = S.Policy(delim=lambda t: t % 6 == 0, sentence_len=2, ar=lambda t: t % 5 == 0, n1=2, replace=True)
    small, large = Stub(0), Stub(500)
    tr = S.speculative_thinking_policy(small, large, [1, 2, 3, 6], 6, pol)       # sentence = ids 4, 5 -> dropped
    assert tr.seq == [1, 2, 3, 6, 504, 505, 6, 7, 8, 9]
    assert tr.actions == [(S.KIND_AR, 5, 2, 4, 4, 2)]
    assert tr.large_feeds == [(0, 4), (4, 5)] and tr.small_truncates == [4]
    assert tr.small_feeds == [(0, 4), (4, 5), (4, 6), (6, 7), (7, 8), (8, 9)]
