"""Oracle of the takeover schedule (test infrastructure only).

Follows the Affirmation/Reflection takeover of Section 3 (1) of the paper: the speculative
(small) model decodes; when a trigger fires on a token it emitted, the target (large) model
first catches up on every token it has not yet seen (the "prefix" pass of Section 4), then
writes a fixed-length segment (n1 tokens, Appendix C), and the small model resumes after
catching up on that segment.  Text keyword matching is replaced by a predicate on token ids.

A model here is any object with `feed(tokens) -> int` (greedy next token after feeding the
tokens at the end of its own cache) so that the schedule can be traced by hand with stubs.
"""
from dataclasses import dataclass, field
from typing import Callable, List, Sequence, Tuple

SMALL, LARGE = 0, 1


@dataclass
class Trace:
    seq: List[int]
    prompt_len: int
    src: List[int] = field(default_factory=list)          # per output token: SMALL or LARGE
    triggers: List[int] = field(default_factory=list)     # absolute positions of trigger tokens
    large_prefill: List[Tuple[int, int]] = field(default_factory=list)   # half-open spans fed to large
    large_decode: List[Tuple[int, int]] = field(default_factory=list)    # positions written by large
    small_prefill: List[Tuple[int, int]] = field(default_factory=list)   # catch-up spans fed to small
    large_decode_feeds: int = 0                                          # single-token feeds to large

    @property
    def modify_ratio(self):
        return sum(1 for s in self.src if s == LARGE) / max(1, len(self.src))


def window_rule(kw: Callable[[int], bool], delim: Callable[[int], bool] = None, window: int = 1):
    """Predicate on (seq, p).  window 1: kw(seq[p]).  window w + 1 >= 2: the w tokens ending at p are the
    sentence after a delimiter -- delim(seq[p-w]), no delimiter among seq[p-w+1 .. p-1] -- and hold a keyword."""
    def fire(seq: Sequence[int], p: int) -> bool:
        if window == 1:
            return kw(seq[p])
        w = window - 1
        if p - w < 0 or not delim(seq[p - w]):
            return False
        if any(delim(t) for t in seq[p - w + 1:p]):
            return False
        return any(kw(t) for t in seq[p - w + 1:p + 1])
    return fire


def speculative_thinking(small, large, prompt: Sequence[int], n_out: int, n_seg: int, fire) -> Trace:
    seq = list(prompt)
    P = len(seq)
    tr = Trace(seq=seq, prompt_len=P)
    if n_out <= 0:
        return tr
    nxt_small = small.feed(seq[:P])
    large.feed(seq[:P])            # target also reads the prompt up front; its prediction is unused
    kv_small = kv_large = P
    while True:
        seq.append(nxt_small)
        tr.src.append(SMALL)
        T = len(seq)
        if T - P == n_out:
            break
        if fire(seq, T - 1):
            tr.triggers.append(T - 1)
            tr.large_prefill.append((kv_large, T))
            nxt_large = large.feed(seq[kv_large:T])
            kv_large = T
            seg_lo = T
            done = False
            for j in range(n_seg):
                seq.append(nxt_large)
                tr.src.append(LARGE)
                if len(seq) - P == n_out:
                    done = True
                    break
                if j < n_seg - 1:                      # the segment's last token is not fed to large yet
                    nxt_large = large.feed([seq[-1]])
                    tr.large_decode_feeds += 1
                    kv_large += 1
            tr.large_decode.append((seg_lo, len(seq)))
            if done:
                break
            T = len(seq)
            tr.small_prefill.append((kv_small, T))
            nxt_small = small.feed(seq[kv_small:T])
            kv_small = T
        else:
            nxt_small = small.feed([seq[-1]])
            kv_small += 1
    return tr


class GreedyModel:
    """Adapter: an OracleModel seen as `feed(tokens) -> greedy token`; keeps every logits vector."""

    def __init__(self, model, keep_logits=False):
        from . import oracle as _o
        self._o = _o
        self.model = model
        self.keep = keep_logits
        self.logits = []          # (kv_len after feed, logits) per feed

    def feed(self, tokens):
        lg = self.model.feed(tokens)
        if self.keep:
            self.logits.append((self.model.kv_len, lg))
        return self._o.argmax(lg)

    def truncate(self, new_len):
        self.model.truncate(new_len)


# ---------------------------------------------------------------------------------------------------
# The full policy of Section 3: (1) Affirmation/Reflection, (2) Verification and (3) Excessive-reflection
# takeovers, with the sentence after a delimiter examined as a window of `sentence_len` tokens
# (Appendix C: n1), the "in place of" (replace) reading of Section 2.2, and the schedule of the
# non-reasoning-speculator variant (Section 4.3 / Appendix: the target writes the first tokens and takes
# over after every delimiter).  Token classes are predicates on ids.
# ---------------------------------------------------------------------------------------------------
AUX = 2
KIND_INITIAL, KIND_AR, KIND_VERIFY, KIND_EXCESS = 0, 1, 2, 3


@dataclass
class Policy:
    delim: Callable[[int], bool]
    sentence_len: int = 1                      # tokens after a delimiter that make up "the sentence"
    ar: Callable[[int], bool] = None           # Affirmation / Reflection keywords -> n1 tokens by the target
    n1: int = 20
    verify: Callable[[int], bool] = None       # verification cues -> n2 tokens by the target
    n2: int = 125
    neg: Callable[[int], bool] = None          # negative (reflection) sentences feed the counter c
    neg_threshold: int = 15                    # an intervention when c exceeds it
    aux: Sequence[int] = ()                    # the auxiliary sentence inserted by that intervention
    n3: int = 125
    replace: bool = False                      # (1) discards the drafted sentence instead of keeping it
    unconditional: bool = False                # every sentence drafted by the speculative model is taken over
    initial_target: int = 0                    # the target writes this many tokens first


@dataclass
class PolicyTrace:
    seq: List[int]
    prompt_len: int
    src: List[int] = field(default_factory=list)             # per output token: SMALL, LARGE or AUX
    actions: List[Tuple[int, int, int, int, int, int]] = field(default_factory=list)
    # (kind, position of the sentence's last token or -1, tokens dropped, aux_lo, aux_hi, tokens granted)
    small_feeds: List[Tuple[int, int]] = field(default_factory=list)     # half-open spans fed to each model,
    large_feeds: List[Tuple[int, int]] = field(default_factory=list)     # in order
    small_truncates: List[int] = field(default_factory=list)
    large_truncates: List[int] = field(default_factory=list)


def speculative_thinking_policy(small, large, prompt: Sequence[int], n_out: int, pol: Policy) -> PolicyTrace:
    """Models need `feed(tokens) -> greedy next token` and, for the replace reading, `truncate(new_len)`."""
    seq = list(prompt)
    P = len(seq)
    tr = PolicyTrace(seq=seq, prompt_len=P)
    if n_out <= 0:
        return tr
    w = pol.sentence_len
    st = dict(kv_s=0, kv_l=0, c=0, start=None, all_small=True, pending=None, pred={})

    def feed(which):
        model, key, log = (small, "kv_s", tr.small_feeds) if which == SMALL else (large, "kv_l", tr.large_feeds)
        lo, hi = st[key], len(seq)
        if hi == lo:                       # nothing new (a replaced sentence right after the prompt): the
            return st["pred"][which]       # prediction made for this position stands
        assert hi > lo
        log.append((lo, hi))
        st[key] = hi
        st["pred"][which] = model.feed(seq[lo:hi])
        return st["pred"][which]

    def done():
        return len(seq) - P >= n_out

    def emit(tok, source):
        """Appends one output token and does the sentence bookkeeping; returns True when the budget is spent."""
        seq.append(tok)
        tr.src.append(source)
        pos = len(seq) - 1
        st["pending"] = None
        if st["start"] is not None:
            if source != SMALL:
                st["all_small"] = False
            if pos == st["start"] + w - 1:                     # the sentence is complete: classify it
                sent = seq[st["start"]:pos + 1]
                kind = None
                if pol.neg is not None and any(pol.neg(t) for t in sent):
                    st["c"] += 1
                    if st["c"] > pol.neg_threshold:
                        st["c"] = 0
                        kind = KIND_EXCESS
                if kind is None and pol.verify is not None and any(pol.verify(t) for t in sent):
                    kind = KIND_VERIFY
                if kind is None and st["all_small"] and (
                        pol.unconditional or (pol.ar is not None and any(pol.ar(t) for t in sent))):
                    kind = KIND_AR
                if kind is not None:
                    st["pending"] = (kind, st["start"], pos)
                st["start"] = None
        if pol.delim(tok):                                     # a delimiter (re)starts the sentence after it
            st["start"], st["all_small"] = pos + 1, True
        return done()

    def insert_aux():
        lo = len(seq)
        for t in pol.aux:
            if emit(t, AUX):
                break
        st["pending"] = None                                   # the inserted sentence triggers nothing itself
        return lo, len(seq)

    def target_segment(n, nxt_known=None):
        """The target writes n tokens (its count restarts if a takeover fires inside); returns small's next token."""
        remaining = n
        nxt = feed(LARGE) if nxt_known is None else nxt_known
        while remaining > 0:
            if emit(nxt, LARGE):
                return None
            remaining -= 1
            act = st["pending"]
            if act is not None:                                # only (2) and (3) can fire on the target's own text
                kind, s0, e0 = act
                if kind == KIND_EXCESS:
                    lo, hi = insert_aux()
                    tr.actions.append((kind, e0, 0, lo, hi, pol.n3))
                    if done():
                        return None
                    remaining = pol.n3
                else:
                    tr.actions.append((kind, e0, 0, len(seq), len(seq), pol.n2))
                    remaining = pol.n2
            if remaining > 0:                                  # the segment's last token is not fed to the target
                nxt = feed(LARGE)
        return feed(SMALL)

    nxt_small = feed(SMALL)
    nxt_large = feed(LARGE)
    if pol.delim(seq[-1]):
        st["start"], st["all_small"] = P, True
    if pol.initial_target > 0:
        tr.actions.append((KIND_INITIAL, -1, 0, P, P, pol.initial_target))
        nxt_small = target_segment(pol.initial_target, nxt_known=nxt_large)
        if nxt_small is None:
            return tr
    while True:
        if emit(nxt_small, SMALL):
            break
        act = st["pending"]
        if act is None:
            nxt_small = feed(SMALL)
            continue
        kind, s0, e0 = act
        if kind == KIND_AR:
            dropped = 0
            if pol.replace:                                    # the drafted sentence goes; the target writes in its place
                dropped = e0 - s0 + 1
                del seq[s0:]
                del tr.src[s0 - P:]
                if st["kv_s"] > s0:
                    small.truncate(s0)
                    tr.small_truncates.append(s0)
                    st["kv_s"] = s0
                if st["kv_l"] > s0:
                    large.truncate(s0)
                    tr.large_truncates.append(s0)
                    st["kv_l"] = s0
            tr.actions.append((kind, e0, dropped, len(seq), len(seq), pol.n1))
            n = pol.n1
        elif kind == KIND_VERIFY:
            tr.actions.append((kind, e0, 0, len(seq), len(seq), pol.n2))
            n = pol.n2
        else:
            lo, hi = insert_aux()
            tr.actions.append((kind, e0, 0, lo, hi, pol.n3))
            if done():
                break
            n = pol.n3
        nxt_small = target_segment(n)
        if nxt_small is None:
            break
    return tr
