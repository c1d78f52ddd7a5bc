"""GPU parity of the batched decode step (independent sequences of ragged length sharing one set of weights)
against one CPU oracle model per sequence."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2504_12329_amd import binding as B, synth
from tests.gpu_common import LOGIT_TOL, print_case, rel_err

pytestmark = pytest.mark.gpu

MIN_MARGIN = 0.008


def _margin(lg):
    s = np.sort(lg)
    return float((s[-1] - s[-2]) / np.abs(lg).max())


def _setup(name, n_seq, seed, max_seq, n_layers=None, gen_device="cpu", max_chunk=64, vocab=None):
    cfg = synth.model_config(name, max_seq=max_seq, max_chunk=max_chunk, n_layers=n_layers)
    if vocab is not None:
        cfg["vocab"] = vocab
    w = synth.make_weights(cfg, seed, device=gen_device)
    oracles = [O.OracleModel(synth.oracle_config(cfg), synth.oracle_views(cfg, w)) for _ in range(n_seq)]
    wg = dict(embed=w["embed"].cuda(), final_norm=w["final_norm"].cuda(),
              lm_head=None if w["lm_head"] is None else w["lm_head"].cuda(),
              layers=[{k: v.cuda() for k, v in lw.items()} for lw in w["layers"]])
    return cfg, B.Batch(cfg, wg, n_seq), oracles


def _run(cfg, batch, oracles, lengths, steps, drop_after=None):
    """Prefills ragged prompts, then `steps` teacher-forced batched steps (both sides follow the oracle's tokens);
    after `drop_after` steps only the even sequences keep going."""
    n = len(oracles)
    worst, checked = 0.0, 0
    toks = []
    for s in range(n):
        prompt = synth.make_prompt(lengths[s], cfg["vocab"], 100 + s)
        lg_o = oracles[s].feed(prompt)
        lg_g, tok_g = batch.prefill(s, prompt)
        worst = max(worst, rel_err(lg_g, lg_o))
        assert tok_g == O.argmax(lg_g)
        toks.append(O.argmax(lg_o))
    active = list(range(n))
    for step in range(steps):
        if drop_after is not None and step == drop_after:
            active = [s for s in active if s % 2 == 0]
        order = active[::-1] if step % 2 else active            # row order must not matter
        lg_g, nxt = batch.decode_step(order, [toks[s] for s in order], want_logits=True)
        for r, s in enumerate(order):
            lg_o = oracles[s].feed([toks[s]])
            worst = max(worst, rel_err(lg_g[r], lg_o))
            assert nxt[r] == O.argmax(lg_g[r])                  # the kernel's arg-max of its own logits
            if _margin(lg_o) >= MIN_MARGIN:
                assert nxt[r] == O.argmax(lg_o)
                checked += 1
            toks[s] = O.argmax(lg_o)
    for s in range(n):
        assert batch.kv_len(s) == oracles[s].kv_len
    print_case("worst relative logit error", worst, "greedy tokens compared", checked)
    return worst


def test_tiny_batch_ragged_lengths():
    print_case("tiny model, 7 sequences of 3..60 tokens, 12 batched steps, 4 sequences leave after 5")
    cfg, batch, oracles = _setup("tiny_small", 7, 1, max_seq=128)
    assert _run(cfg, batch, oracles, [3, 60, 17, 33, 1, 48, 64], 12, drop_after=5) <= LOGIT_TOL
    # a truncated sequence continues from its shorter cache, alone in the batch
    oracles[2].truncate(10)
    batch.truncate(2, 10)
    lg_o = oracles[2].feed([5])
    lg_g, nxt = batch.decode_step([2], [5], want_logits=True)
    assert rel_err(lg_g[0], lg_o) <= LOGIT_TOL and batch.kv_len(2) == 11
    batch.close()


def test_tiny_batch_vocabulary_not_a_multiple_of_four():
    """1022 logits per row: the batched arg-max and the LM-head partials take their element-by-element paths, and
    the last arg-max segment is ragged."""
    print_case("tiny model, vocabulary 1022, 5 sequences, 6 batched steps")
    cfg, batch, oracles = _setup("tiny_small", 5, 3, max_seq=128, vocab=1022)
    assert _run(cfg, batch, oracles, [9, 40, 2, 64, 21], 6) <= LOGIT_TOL
    batch.close()


@pytest.mark.parametrize("name,layers,lens", [
    ("tiny_small", None, [1 + (7 * i) % 60 for i in range(40)]),
    ("qwen1p5b", 1, [5 + (97 * i) % 700 for i in range(40)])])
def test_row_bits_do_not_depend_on_the_batch(name, layers, lens):
    """A sequence's logits of a batched step are the same bits whether it decodes alone, with two others, with 16,
    32 or 39 others, and wherever its row sits: the K slices of the step's GEMMs do not follow the row count."""
    n = len(lens)
    cfg, batch, _ = _setup(name, n, 5, max_seq=800, n_layers=layers, gen_device="cuda" if layers else "cpu")
    toks = []
    for s in range(n):
        prompt = synth.make_prompt(lens[s], cfg["vocab"], 700 + s)
        for lo in range(0, lens[s], 64):
            batch.prefill(s, prompt[lo:lo + 64], want_logits=False)
        toks.append(int(prompt[-1]))
    full, nxt_full = batch.decode_step(list(range(n)), toks, want_logits=True)
    full = np.array(full, copy=True)
    for group in ([3], [5, 3, 1], list(range(17)), list(range(4, 37)), list(range(n))[::-1]):
        for s in group:
            batch.truncate(s, lens[s])
        lg, nxt = batch.decode_step(group, [toks[s] for s in group], want_logits=True)
        for r, s in enumerate(group):
            assert np.array_equal(np.asarray(lg[r]).view(np.uint32), full[s].view(np.uint32)), (len(group), s)
            assert nxt[r] == nxt_full[s]
    print_case(name, "rows per step compared", [1, 3, 17, 33, n])
    batch.close()


def test_batch_crosses_attention_ranges():
    """One layer at the 1.5B shape: sequences of 30, 700 and 1030 keys decode together (1, 11 and 17 key ranges)."""
    print_case("1.5B shape, 1 layer: 3 sequences of 30 / 700 / 1030 tokens, 3 batched steps")
    cfg, batch, oracles = _setup("qwen1p5b", 3, 8, max_seq=1100, n_layers=1, gen_device="cuda")
    lengths = [30, 700, 1030]
    toks = []
    for s in range(3):
        prompt = synth.make_prompt(lengths[s], cfg["vocab"], 200 + s)
        lg_o = None
        for lo in range(0, lengths[s], 64):
            chunk = prompt[lo:lo + 64]
            lg_o = oracles[s].feed(chunk)
            lg_g, _ = batch.prefill(s, chunk)
        assert rel_err(lg_g, lg_o) <= LOGIT_TOL
        toks.append(O.argmax(lg_o))
    worst = 0.0
    for step in range(3):
        lg_g, nxt = batch.decode_step([0, 1, 2], toks, want_logits=True)
        for s in range(3):
            lg_o = oracles[s].feed([toks[s]])
            worst = max(worst, rel_err(lg_g[s], lg_o))
            toks[s] = O.argmax(lg_o)
    print_case("worst relative logit error", worst)
    assert worst <= LOGIT_TOL
    batch.close()


def test_batch_argument_errors():
    cfg, batch, oracles = _setup("tiny_small", 3, 1, max_seq=16)
    with pytest.raises(B.StError):
        batch.decode_step([0, 0], [1, 2])                       # a sequence twice in one step
    with pytest.raises(B.StError):
        batch.decode_step([3], [1])                             # no such sequence
    with pytest.raises(B.StError):
        batch.decode_step([0], [cfg["vocab"]])                  # token outside the vocabulary
    batch.prefill(1, synth.make_prompt(16, cfg["vocab"], 1), want_logits=False)
    with pytest.raises(B.StError) as e:
        batch.decode_step([1], [1])                             # cache full
    assert e.value.code == B.ST_ERANGE and batch.kv_len(1) == 16 and batch.kv_len(0) == 0
    with pytest.raises(B.StError):
        B.Batch(cfg, batch.weights, 65)                         # more sequences than the step supports
    batch.close()


# (prompt seed, prompt length): searched on the CPU so that the oracle's own run of each sequence (mod-16 rule, 48
# outputs, segments of 8) keeps every top-1/top-2 logit gap above MIN_MARGIN; re-checked below
LOOP_PROMPTS = [(460, 28), (537, 47), (591, 25), (681, 15), (962, 22), (966, 10)]


def test_batched_loop_matches_per_sequence_oracle():
    """Six sequences of different prompt length run the two-model loop together; each must reproduce the schedule
    oracle's single-sequence trace (tokens and who wrote them)."""
    from oracle import schedule as S
    n = len(LOOP_PROMPTS)
    cfg, bs, o_small = _setup("tiny_small", n, 1, max_seq=128)
    _, bl, o_large = _setup("tiny_large", n, 2, max_seq=128)
    V = cfg["vocab"]
    fire = S.window_rule(lambda t: t % 16 == 0)
    prompts, traces = [], []
    for i, (seed, plen) in enumerate(LOOP_PROMPTS):
        prompt = synth.make_prompt(plen, V, seed)
        a, b = S.GreedyModel(o_small[i], keep_logits=True), S.GreedyModel(o_large[i], keep_logits=True)
        tr = S.speculative_thinking(a, b, prompt, 48, 8, fire)
        margin = min(_margin(lg) for g in (a, b) for _, lg in g.logits)
        assert margin >= MIN_MARGIN, f"sequence {i}: oracle run has a near-tie ({margin:.4f}); pick another seed"
        prompts.append(prompt)
        traces.append(tr)
    out = B.st_generate_batch(bs, bl, prompts, 48, 8, V, kw=B.host_bitmap(V, range(0, V, 16)))
    total_large = 0
    for i, tr in enumerate(traces):
        assert out["seqs"][i].tolist() == tr.seq, i
        assert out["srcs"][i][:48].tolist() == tr.src, i
        assert bs.kv_len(i) == o_small[i].kv_len and bl.kv_len(i) == o_large[i].kv_len
        total_large += sum(tr.src)
    print_case("hand-overs per sequence", [len(tr.triggers) for tr in traces])
    assert out["stats"]["n_out"] == 48 * n and out["stats"]["n_large"] == total_large
    assert out["stats"]["n_handoffs"] == sum(len(tr.triggers) for tr in traces)
    bs.close()
    bl.close()


FORCED_PROMPTS = [(305, 23, 0), (355, 13, 2), (358, 34, 3), (408, 24, 5)]   # prompt seed, length, start of the count


def test_batched_loop_with_staggered_forced_period():
    """Forced hand-overs every 6th speculative token, each sequence starting its count elsewhere: the two models
    then work on different sequences at the same time; every sequence still reproduces its own oracle trace,
    whatever the gather threshold (scheduling changes when a token is computed, never which)."""
    from oracle import schedule as S
    n = len(FORCED_PROMPTS)
    cfg, bs, o_small = _setup("tiny_small", n, 1, max_seq=128)
    _, bl, o_large = _setup("tiny_large", n, 2, max_seq=128)
    V = cfg["vocab"]
    prompts, traces = [], []
    for i, (seed, plen, phase) in enumerate(FORCED_PROMPTS):
        prompt = synth.make_prompt(plen, V, seed)
        a, b = S.GreedyModel(o_small[i], keep_logits=True), S.GreedyModel(o_large[i], keep_logits=True)
        count = {"n": phase}

        def fire(seq, p, count=count):
            count["n"] += 1
            return count["n"] % 6 == 0
        tr = S.speculative_thinking(a, b, prompt, 40, 4, fire)
        margin = min(_margin(lg) for g in (a, b) for _, lg in g.logits)
        assert margin >= MIN_MARGIN, f"sequence {i}: oracle run has a near-tie ({margin:.4f}); pick another seed"
        prompts.append(prompt)
        traces.append(tr)
    with pytest.raises(B.StError, match="forced_phase"):     # rejected before anything is launched
        B.st_generate_batch(bs, bl, prompts, 40, 4, V, forced_period=6, forced_phase=[0, -1, 0, 0])
    phases = [p for _, _, p in FORCED_PROMPTS]
    for gather in (0, 3, n):        # at once / held until three wait / held until nothing else can run
        for i in range(n):
            bs.truncate(i, 0)
            bl.truncate(i, 0)
        out = B.st_generate_batch(bs, bl, prompts, 40, 4, V, forced_period=6, forced_phase=phases, gather=gather)
        for i, tr in enumerate(traces):
            assert out["seqs"][i].tolist() == tr.seq, (gather, i)
            assert out["srcs"][i][:40].tolist() == tr.src, (gather, i)
        assert out["stats"]["n_handoffs"] == sum(len(tr.triggers) for tr in traces)
    with pytest.raises(B.StError, match="gather"):
        B.st_generate_batch(bs, bl, prompts, 40, 4, V, forced_period=6, gather=n + 1)
    bs.close()
    bl.close()


def _ragged_against_oracles(cfg, batch, oracles, cached, lens, decode_after=True):
    """Sequence j holds cached[j] tokens; one ragged pass feeds lens[j] more to each (segments in reverse order); every
    sequence's last-position logits against its own oracle, then one batched decode step over all of them."""
    n = len(lens)
    for j in range(n):
        if cached[j]:
            pre = synth.make_prompt(cached[j], cfg["vocab"], 300 + j)
            oracles[j].feed(pre)
            batch.prefill(j, pre, want_logits=False)
    chunks = [synth.make_prompt(lens[j], cfg["vocab"], 400 + j) for j in range(n)]
    order = list(range(n))[::-1]
    lg_g, nxt = batch.prefill_many(order, [chunks[j] for j in order], want_logits=True)
    worst, toks = 0.0, {}
    for r, j in enumerate(order):
        lg_o = oracles[j].feed(chunks[j])
        worst = max(worst, rel_err(lg_g[r], lg_o))
        assert nxt[r] == O.argmax(lg_g[r]) and batch.kv_len(j) == oracles[j].kv_len
        toks[j] = O.argmax(lg_o)
    if decode_after:
        lg_g, _ = batch.decode_step(list(range(n)), [toks[j] for j in range(n)], want_logits=True)
        for j in range(n):
            worst = max(worst, rel_err(lg_g[j], oracles[j].feed([toks[j]])))
    print_case("worst relative logit error", worst)
    return worst


def test_ragged_catch_up_of_sixteen_sequences():
    """Sixteen segments of 1..40 rows on caches of 0..150 tokens in one pass: the attention of the pass is one launch
    whose blocks find their segment in a device table (several key splits, segments shorter than a row block, an
    empty cache among them)."""
    rng = np.random.default_rng(77)
    lens = [int(v) for v in rng.integers(1, 41, 16)]
    cached = [int(v) for v in rng.integers(0, 151, 16)]
    cached[3], lens[3], lens[9] = 0, 1, 40
    print_case("tiny model, 16 sequences: ragged catch-up of", lens, "tokens onto caches of", cached)
    cfg, batch, oracles = _setup("tiny_small", 16, 1, max_seq=256, max_chunk=512)
    assert _ragged_against_oracles(cfg, batch, oracles, cached, lens) <= LOGIT_TOL
    batch.close()


@pytest.mark.parametrize("lens,cached,f16", [([40, 130, 7], [90, 20, 300], False), ([150, 200], [0, 64], False),
                                             ([40, 130, 7], [90, 20, 300], True)])
def test_ragged_catch_up_pass_head_dim_128(lens, cached, f16):
    """The same at head_dim 128 (1.5B shape, 2 layers), whose attention kernel is a different one: a pass of 177 rows
    (two-term queries, streaming GEMMs -- or, with the fp16 weight copy attached, the ring GEMMs on fp16 operands)
    and one of 350 rows (256 x 256 tiles)."""
    print_case("1.5B shape, 2 layers: ragged catch-up of", lens, "tokens onto caches of", cached,
               "(fp16 operand mode)" if f16 else "")
    cfg, batch, oracles = _setup("qwen1p5b", len(lens), 6, max_seq=512, n_layers=2, gen_device="cuda", max_chunk=512)
    if f16:
        batch.attach_f16()
    assert _ragged_against_oracles(cfg, batch, oracles, cached, lens) <= LOGIT_TOL
    batch.close()


@pytest.mark.parametrize("lens", [[5, 1, 33, 12], [70, 90, 60], [200, 150, 100]])
def test_ragged_catch_up_pass(lens):
    """Several sequences with different cached lengths each receive a chunk of a different length in one pass
    (the short-chunk, 129..256-row and long-chunk GEMM regimes by total rows); each sequence's last-position logits must match
    its own oracle, and a batched decode step afterwards must see the appended keys."""
    n = len(lens)
    print_case("tiny model, ragged catch-up of", lens, "tokens onto caches of", [7 * (j + 1) for j in range(n)])
    cfg, batch, oracles = _setup("tiny_small", n + 1, 1, max_seq=320, max_chunk=512)
    for j in range(n):                                    # different cached lengths first (sequence n stays empty)
        pre = synth.make_prompt(7 * (j + 1), cfg["vocab"], 300 + j)
        oracles[j].feed(pre)
        batch.prefill(j, pre, want_logits=False)
    chunks = [synth.make_prompt(lens[j], cfg["vocab"], 400 + j) for j in range(n)]
    order = list(range(n))[::-1]                          # the order of the segments must not matter
    lg_g, nxt = batch.prefill_many(order, [chunks[j] for j in order], want_logits=True)
    worst, toks = 0.0, {}
    for r, j in enumerate(order):
        lg_o = oracles[j].feed(chunks[j])
        worst = max(worst, rel_err(lg_g[r], lg_o))
        assert nxt[r] == O.argmax(lg_g[r]) and batch.kv_len(j) == oracles[j].kv_len
        toks[j] = O.argmax(lg_o)
    lg_g, _ = batch.decode_step(list(range(n)), [toks[j] for j in range(n)], want_logits=True)
    for j in range(n):
        worst = max(worst, rel_err(lg_g[j], oracles[j].feed([toks[j]])))
    print_case("worst relative logit error", worst)
    assert worst <= LOGIT_TOL and batch.kv_len(n) == 0
    batch.close()
