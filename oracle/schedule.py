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
    """Predicate on (seq, p): kw(seq[p]) and, for window 2, p >= 1 and delim(seq[p-1])."""
    def fire(seq: Sequence[int], p: int) -> bool:
        if not kw(seq[p]):
            return False
        if window == 1:
            return True
        return p >= 1 and delim(seq[p - 1])
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
