"""GPU parity of the full takeover policy (st_generate_policy) on the tiny model pair against the schedule oracle
driven by the CPU oracle models: identical tokens, sources and takeover records."""
import numpy as np
import pytest

from oracle import schedule as S
from paper_2504_12329_amd import binding as B, synth
from tests.gpu_common import make_pair, print_case

pytestmark = pytest.mark.gpu

MIN_MARGIN = 0.008   # see tests/test_gpu_tiny.py: prompt seeds were searched on the CPU for this top-1/top-2 gap
V = 1024


def _ids(pred):
    return [t for t in range(V) if pred(t)]


# name -> (prompt seed, outputs, oracle policy, keyword arguments of the library call)
SCENARIOS = {
    "replace": (392, 48,
                S.Policy(delim=lambda t: t % 5 == 0, sentence_len=3, ar=lambda t: t % 4 == 0, n1=6, replace=True),
                dict(delim=_ids(lambda t: t % 5 == 0), sentence_len=3, ar=_ids(lambda t: t % 4 == 0), n1=6,
                     replace=True)),
    "verify_excess": (663, 56,
                      S.Policy(delim=lambda t: t % 5 == 0, sentence_len=2, verify=lambda t: t % 7 == 0, n2=9,
                               neg=lambda t: t % 3 == 0, neg_threshold=1, aux=(11, 22, 33), n3=7,
                               ar=lambda t: t % 4 == 0, n1=5),
                      dict(delim=_ids(lambda t: t % 5 == 0), sentence_len=2, verify=_ids(lambda t: t % 7 == 0), n2=9,
                           neg=_ids(lambda t: t % 3 == 0), neg_threshold=1, aux=(11, 22, 33), n3=7,
                           ar=_ids(lambda t: t % 4 == 0), n1=5)),
    "nonreasoning": (969, 48,
                     S.Policy(delim=lambda t: t % 4 == 0, sentence_len=1, unconditional=True, n1=4, initial_target=10),
                     dict(delim=_ids(lambda t: t % 4 == 0), sentence_len=1, unconditional=True, n1=4,
                          initial_target=10)),
}


@pytest.fixture(scope="module")
def pair():
    cfg, gs, os_ = make_pair("tiny_small", 1, max_seq=256, max_chunk=64)
    _, gl, ol = make_pair("tiny_large", 2, max_seq=256, max_chunk=64)
    yield cfg, gs, os_, gl, ol
    gs.close()
    gl.close()


@pytest.mark.parametrize("name", sorted(SCENARIOS))
def test_policy_matches_oracle(pair, name):
    cfg, gs, os_, gl, ol = pair
    seed, n_out, pol, kw = SCENARIOS[name]
    prompt = synth.make_prompt(32, cfg["vocab"], seed)
    os_.truncate(0)
    ol.truncate(0)
    a, b = S.GreedyModel(os_, keep_logits=True), S.GreedyModel(ol, keep_logits=True)
    tr = S.speculative_thinking_policy(a, b, prompt, n_out, pol)
    margin = min((np.sort(lg)[-1] - np.sort(lg)[-2]) / np.abs(lg).max() for g in (a, b) for _, lg in g.logits)
    assert margin >= MIN_MARGIN, f"oracle run has a near-tie (margin {margin:.4f}); pick another prompt seed"
    kinds = [act[0] for act in tr.actions]
    print_case(name, "actions", tr.actions)
    if name == "replace":
        assert any(act[2] > 0 for act in tr.actions)
    if name == "verify_excess":
        assert S.KIND_VERIFY in kinds and S.KIND_EXCESS in kinds and S.AUX in tr.src
    if name == "nonreasoning":
        assert kinds[0] == S.KIND_INITIAL and kinds.count(S.KIND_AR) >= 3
    gs.truncate(0)
    gl.truncate(0)
    bm = {k: B.host_bitmap(V, v) for k, v in kw.items() if k in ("delim", "ar", "verify", "neg")}
    rest = {k: v for k, v in kw.items() if k not in bm}
    out = B.st_generate_policy(gs, gl, prompt, n_out, V, **bm, **rest)
    assert out["seq"].tolist() == tr.seq
    assert out["src"].tolist() == tr.src
    assert out["actions"] == tr.actions
    assert out["stats"]["n_out"] == n_out and out["stats"]["n_handoffs"] == len(tr.actions)
    assert out["stats"]["n_large"] == tr.src.count(S.LARGE)
    assert gs.kv_len == os_.kv_len and gl.kv_len == ol.kv_len          # both sides fed the same spans


def test_policy_argument_errors(pair):
    cfg, gs, os_, gl, ol = pair
    gs.truncate(0)
    gl.truncate(0)
    prompt = synth.make_prompt(8, V, 1)
    d = B.host_bitmap(V, [0])
    with pytest.raises(B.StError):
        B.st_generate_policy(gs, gs, prompt, 4, V, delim=d)                       # same model twice
    with pytest.raises(B.StError):
        B.st_generate_policy(gs, gl, prompt, 4, V, delim=None)                    # no delimiter class
    with pytest.raises(B.StError):
        B.st_generate_policy(gs, gl, prompt, 4, V, delim=d, sentence_len=0)
    with pytest.raises(B.StError):
        B.st_generate_policy(gs, gl, prompt, 4, V, delim=d, neg=d, aux=(V,))      # auxiliary token out of range
    with pytest.raises(B.StError):
        B.st_generate_policy(gs, gl, prompt, 300, V, delim=d)                     # exceeds max_seq
    assert gs.kv_len == 0 and gl.kv_len == 0
