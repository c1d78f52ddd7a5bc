"""GPU parity at the paper's model shapes (1.5B whole, 7B- and 32B-shaped layer subsets) against the
oracle, and cross-path properties at sizes the oracle cannot reach."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2504_12329_amd import binding as B, synth
from tests.gpu_common import LOGIT_TOL, make_pair, print_case, rel_err

pytestmark = pytest.mark.gpu

MIN_MARGIN = 0.008
FAST_TOL = 2 * LOGIT_TOL   # opt-in passes with single-bf16 inputs (ST_PREFILL_FAST): about twice the default error


def _margin(lg):
    s = np.sort(lg)
    return float((s[-1] - s[-2]) / np.abs(lg).max())


def _teacher_forced(cfg, g, o, prompt, splits, n_decode, fast=False):
    """Feeds `prompt` in the given chunk sizes, then n_decode oracle-chosen tokens one by one."""
    worst = 0.0
    lo = hi = 0
    for n in splits:
        hi = lo + n
        lg_g, tok_g = g.prefill(prompt[lo:hi], fast=fast)
        lo = hi
    assert hi == len(prompt)
    lg_o = o.feed(prompt)
    worst = max(worst, rel_err(lg_g, lg_o))
    checked = 0
    for _ in range(n_decode):
        if _margin(lg_o) >= MIN_MARGIN:
            assert tok_g == O.argmax(lg_o)
            checked += 1
        assert tok_g == O.argmax(lg_g)
        tok = O.argmax(lg_o)
        lg_o = o.feed([tok])
        lg_g, tok_g = g.decode_step(tok)
        worst = max(worst, rel_err(lg_g, lg_o))
    print_case("worst relative logit error", worst, "tokens compared", checked)
    return worst


def test_qwen1p5b_whole_model():
    """The whole 28-layer model: logits within the tolerance at the prompt's end and at each of 32 teacher-forced
    decode steps, and the GPU's greedy token equal to the oracle's at every step whose top-two logit gap in the
    oracle exceeds MIN_MARGIN (a bf16 path may legitimately break a nearer tie the other way)."""
    print_case("1.5B shape, 28 layers: prefill 33+7 tokens, 32 decode steps")
    cfg, g, o = make_pair("qwen1p5b", 1, max_seq=80, max_chunk=48, gen_device="cuda")
    prompt = synth.make_prompt(40, cfg["vocab"], 3)
    assert _teacher_forced(cfg, g, o, prompt, [33, 7], 32) <= LOGIT_TOL
    g.close()


def test_qwen7b_shaped_layers():
    print_case("7B shape (7 query heads per kv head), 2 layers: prefill 37 tokens, 4 decode steps")
    cfg, g, o = make_pair("qwen7b", 4, max_seq=64, max_chunk=64, n_layers=2, gen_device="cuda")
    prompt = synth.make_prompt(37, cfg["vocab"], 5)
    assert _teacher_forced(cfg, g, o, prompt, [37], 4) <= LOGIT_TOL
    g.close()


def test_qwen32b_shaped_layers_prefill_on_existing_cache():
    print_case("32B shape, 2 layers: 70 cached tokens, catch-up chunk of 150 (128 + 22), 3 decode steps")
    cfg, g, o = make_pair("qwen32b", 2, max_seq=256, max_chunk=256, n_layers=2, gen_device="cuda")
    prompt = synth.make_prompt(220, cfg["vocab"], 6)
    assert _teacher_forced(cfg, g, o, prompt, [70, 150], 3) <= LOGIT_TOL
    g.close()


def test_decode_and_prefill_paths_agree_at_long_context():
    """At 4096 + 1024 tokens the oracle is out of reach; the GEMV/split-K decode path and the
    MFMA/flash prefill path are two independent kernel sets and must agree with each other (each
    carries its own bf16 rounding, so the bar is the same as against the oracle)."""
    print_case("1.5B shape, 4 layers: 4096 cached + 1024-token chunk, decode vs prefill of the next tokens")
    cfg = synth.model_config("qwen1p5b", max_seq=5400, max_chunk=1024, n_layers=4)
    w = synth.make_weights(cfg, 1, device="cuda")
    g = B.Model(cfg, w)
    toks = synth.make_prompt(5200, cfg["vocab"], 7)
    g.prefill(toks[:4096], want_logits=False)
    a, _ = g.prefill(toks[4096:5120])                     # one 1024-row chunk on top of 4096 cached keys
    g.truncate(4096)
    g.prefill(toks[4096:4600], want_logits=False)          # same tokens, ragged chunks
    b, _ = g.prefill(toks[4600:5120])
    assert rel_err(b, a) <= LOGIT_TOL
    g.truncate(5119)
    c, _ = g.decode_step(int(toks[5119]))                 # last token again, through the decode kernels
    assert rel_err(c, a) <= LOGIT_TOL
    for i in range(5120, 5124):                           # and a few more, decode vs single-row prefill
        d, _ = g.decode_step(int(toks[i]))
        g.truncate(i)
        e, _ = g.prefill(toks[i:i + 1])
        assert rel_err(e, d) <= LOGIT_TOL
    g.close()


def test_split_attention_matches_oracle_over_many_ranges():
    """One layer, 1.5B shape, 700 cached keys: the decode attention splits them over 11 ranges."""
    print_case("1.5B shape, 1 layer: 700 tokens then 3 decode steps")
    cfg, g, o = make_pair("qwen1p5b", 8, max_seq=720, max_chunk=512, n_layers=1, gen_device="cuda")
    prompt = synth.make_prompt(700, cfg["vocab"], 9)
    assert _teacher_forced(cfg, g, o, prompt, [512, 188], 3) <= LOGIT_TOL
    g.close()


@pytest.mark.parametrize("m,fast", [(32, False), (33, False), (64, False), (65, False), (128, False), (129, False),
                                    (200, False), (256, False), (257, False), (512, False), (513, False),
                                    (129, True), (192, True), (193, True), (257, True), (513, True)])
def test_prefill_kernel_regime_boundaries(m, fast):
    """Chunk lengths on both sides of every kernel switch (one more 32-row activation tile, 128- to 64-byte row
    segments above 128 rows, the streaming kernel up to 240 rows, 256x256 tiles above -- with two-term inputs by
    default; with single bf16 inputs on request: one-term streaming kernel from 129 rows, tiles from 193), on top of
    100 cached keys, against the oracle (2 layers)."""
    print_case(f"1.5B shape, 2 layers: 100 cached + chunk of {m}" + (" (single-term inputs)" if fast else ""))
    cfg, g, o = make_pair("qwen1p5b", 11, max_seq=640, max_chunk=520, n_layers=2, gen_device="cuda")
    prompt = synth.make_prompt(100 + m, cfg["vocab"], 12)
    assert _teacher_forced(cfg, g, o, prompt, [100, m], 1, fast=fast) <= LOGIT_TOL
    g.close()


@pytest.mark.parametrize("fast", [False, True])
@pytest.mark.parametrize("name", ["qwen32b", "qwen7b"])
def test_4096_row_chunk_agrees_with_1024_row_chunks(name, fast):
    """A 4096-row pass has more 256 x 256 output tiles than compute units in the O / down projections (32B shape)
    or the QKV projection (7B shape); the columns left over after whole rounds are cut into K slices of their own,
    which 1024-row passes never do.  Same tokens, both ways, on 300 cached keys (2 layers; the oracle is out of
    reach at this size, the 1024-row path is checked against it in the tests above)."""
    print_case(f"{name} shape, 2 layers: 300 cached + 4096 tokens as one chunk and as four" +
               (" (single-term inputs)" if fast else ""))
    cfg = synth.model_config(name, max_seq=4500, max_chunk=4096, n_layers=2)
    g = B.Model(cfg, synth.make_weights(cfg, 21, device="cuda"))
    toks = synth.make_prompt(4400, cfg["vocab"], 22)
    g.prefill(toks[:300], want_logits=False)
    a, ta = g.prefill(toks[300:4396], fast=fast)
    g.truncate(300)
    for lo in range(300, 4396 - 1024, 1024):
        g.prefill(toks[lo:lo + 1024], want_logits=False, fast=fast)
    b, tb = g.prefill(toks[3372:4396], fast=fast)
    err = rel_err(a, b)
    print_case("relative logit difference", err)
    assert err <= LOGIT_TOL
    c, _ = g.decode_step(int(toks[4396]))                 # the caches the two ways left behind agree as well
    g.truncate(300)
    g.prefill(toks[300:4396], want_logits=False, fast=fast)
    d, _ = g.decode_step(int(toks[4396]))
    assert rel_err(c, d) <= LOGIT_TOL
    g.close()


@pytest.mark.parametrize("fast", [False, True])
def test_4096_row_chunk_tail_tiles_against_oracle(fast):
    """A one-layer model sized so that one 4096-row pass takes every leftover-tile path of the long-chunk GEMM with
    ragged edges, small enough for the oracle: hidden 4288 (17 column tiles of 256, the last 192 wide: one round
    of 256 tiles + 16 tail tiles cut into K slices, in the O and the down projection) and intermediate 2240 (18
    column tiles of 128, the last 64 wide: 256 full tiles + 3 half-width tiles in the fused gate/up GEMM)."""
    print_case("custom shape (hidden 4288, intermediate 2240, 6 q heads per kv head), 1 layer: 40 cached + 4096-row chunk" +
               (" (single-term inputs)" if fast else ""))
    cfg, g, o = make_pair("qwen1p5b", 31, max_seq=4200, max_chunk=4096, n_layers=1, gen_device="cuda",
                          hidden=4288, intermediate=2240, n_q_heads=6, n_kv_heads=1, vocab=2048)
    prompt = synth.make_prompt(4136, cfg["vocab"], 32)
    assert _teacher_forced(cfg, g, o, prompt, [40, 4096], 2, fast=fast) <= LOGIT_TOL
    g.close()


def test_prefill_is_bit_reproducible():
    """Split-K partial sums and split-key attention are merged in fixed orders: same input, same bits."""
    cfg = synth.model_config("qwen1p5b", max_seq=1400, max_chunk=1024, n_layers=2)
    g = B.Model(cfg, synth.make_weights(cfg, 3, device="cuda"))
    toks = synth.make_prompt(1300, cfg["vocab"], 4)
    outs = []
    for _ in range(3):
        g.truncate(0)
        g.prefill(toks[:900], want_logits=False)          # 256x256 tiles
        a, _ = g.prefill(toks[900:1121])                  # 221 rows: two-term path, key splits
        b, _ = g.prefill(toks[1121:1142])                 # 21 rows: small tiles, many K slices
        outs.append((a, b))
    for a, b in outs[1:]:
        assert np.array_equal(a, outs[0][0]) and np.array_equal(b, outs[0][1])
    g.close()


def test_kv_capacity_edge_and_long_decode_buckets():
    """Fill the cache to its last position through both paths; decode across attention-grid buckets."""
    cfg, g, o = make_pair("qwen1p5b", 13, max_seq=1100, max_chunk=512, n_layers=1, gen_device="cuda")
    toks = synth.make_prompt(1100, cfg["vocab"], 14)
    g.prefill(toks[:1020], want_logits=False)
    o.feed(toks[:1020])
    worst = 0.0
    for i in range(1020, 1099):                           # crosses the 1024-key bucket boundary
        lg, _ = g.decode_step(int(toks[i]), want_logits=(i % 13 == 0 or i > 1090))
        lo = o.feed(toks[i:i + 1])
        if lg is not None:
            worst = max(worst, rel_err(lg, lo))
    lg, _ = g.prefill(toks[1099:1100])                    # the very last position, through the prefill path
    worst = max(worst, rel_err(lg, o.feed(toks[1099:1100])))
    assert worst <= LOGIT_TOL and g.kv_len == 1100
    with pytest.raises(B.StError):
        g.decode_step(1)
    g.close()


def test_qwen32b_full_depth_paths_agree():
    """All 64 layers of the 32B shape (65 GB of weights, beyond the oracle's reach): the same position computed
    through the decode kernels, through a one-row catch-up and through a 21-row catch-up (three kernel sets with
    their own bf16 roundings) must agree to the tolerance each is held to against the oracle, and so must the
    greedy continuation where the logit gap allows."""
    print_case("32B shape, 64 layers: 200 cached tokens, position 200 through decode / 1-row / 21-row passes")
    cfg = synth.model_config("qwen32b", max_seq=320, max_chunk=288)
    w = synth.make_weights(cfg, 2, device="cuda")
    g = B.Model(cfg, w)
    toks = synth.make_prompt(201, cfg["vocab"], 21)
    g.prefill(toks[:120], want_logits=False)               # 120 rows: four activation tiles
    g.prefill(toks[120:200], want_logits=False)            # 80 rows: three
    a, tok_a = g.decode_step(int(toks[200]))               # GEMV path
    g.truncate(200)
    b, tok_b = g.prefill(toks[200:201])                    # one-row catch-up
    g.truncate(180)
    c, tok_c = g.prefill(toks[180:201])                    # 21-row catch-up re-deriving the last 20 cache rows
    print_case("decode vs 1-row", rel_err(b, a), "decode vs 21-row", rel_err(c, a), "1-row vs 21-row", rel_err(c, b),
               "margin", _margin(a))
    assert max(rel_err(b, a), rel_err(c, a), rel_err(c, b)) <= LOGIT_TOL
    if _margin(a) >= MIN_MARGIN:
        assert tok_a == tok_b == tok_c
    # A 260-row catch-up at full depth, four ways: two bf16 terms (ring kernels), passes of at most 128 rows
    # (streaming kernel, two terms), fp16 operands (the fp16 weight copy; the QKV input stays in two bf16 terms) and
    # single bf16 operands (ST_PREFILL_FAST).  They share the first 21 cached rows and are compared with the decode
    # step's logits for the same position (the oracle cannot reach this depth).  The three default-precision forms
    # must agree with it to the tolerance; the single-bf16 pass is printed and only has to be the farthest (measured
    # 6.8e-2: through 64 layers of random weights its rounding is amplified past its 4e-2 bound at oracle depths).
    toks = synth.make_prompt(281, cfg["vocab"], 22)
    g.truncate(0)
    g.prefill(toks[:21], want_logits=False)
    two, _ = g.prefill(toks[21:281])
    g.truncate(280)
    dec, _ = g.decode_step(int(toks[280]))
    g.truncate(21)
    g.prefill(toks[21:149], want_logits=False)
    g.prefill(toks[149:277], want_logits=False)
    short, _ = g.prefill(toks[277:281])
    g.truncate(21)
    fast, _ = g.prefill(toks[21:281], fast=True)
    g.attach_f16()
    g.truncate(21)
    f16, _ = g.prefill(toks[21:281])
    print_case("260-row pass against the decode step: two bf16 terms", rel_err(two, dec), "short passes", rel_err(short, dec),
               "fp16 operands", rel_err(f16, dec), "single bf16", rel_err(fast, dec))
    assert max(rel_err(two, dec), rel_err(short, dec), rel_err(f16, dec)) <= LOGIT_TOL
    assert rel_err(fast, dec) > rel_err(f16, dec)
    g.close()


def test_qwen1p5b_long_chunk_at_full_depth():
    """A 300-token prompt through all 28 layers, against the oracle.  Fed as one pass it takes the long-chunk
    kernels; by default their GEMM and attention inputs are two bf16 terms, which leaves the bf16 K/V cache as the
    pass's only rounding, and the pass is held to the same tolerance as everything else -- as are the same prompt in
    passes of at most 256 rows (ST_PREFILL_TWO_TERM) and the decode step that follows.  With ST_PREFILL_FAST the
    inputs are single bf16 numbers: that rounding, amplified through the depth of a random-weight model, about
    doubles the error; it is bounded here so that a regression of the opt-in path still shows."""
    print_case("1.5B shape, 28 layers: 300-token prompt as one pass (default and single-term), as <=256-row passes, then one decode step")
    cfg, g, o = make_pair("qwen1p5b", 1, max_seq=320, max_chunk=300, gen_device="cuda")
    toks = synth.make_prompt(301, cfg["vocab"], 21)
    ref = o.feed(toks[:300])
    one, _ = g.prefill(toks[:300])
    dec, _ = g.decode_step(int(toks[300]))
    ref_dec = o.feed(toks[300:301])
    g.truncate(0)
    two, _ = g.prefill(toks[:300], two_term=True)
    g.truncate(0)
    fast, _ = g.prefill(toks[:300], fast=True)
    print_case("one pass", rel_err(one, ref), "decode after it", rel_err(dec, ref_dec), "<=256-row passes",
               rel_err(two, ref), "one pass, single-term inputs", rel_err(fast, ref))
    assert g.kv_len == 300
    assert rel_err(one, ref) <= LOGIT_TOL and rel_err(two, ref) <= LOGIT_TOL and rel_err(dec, ref_dec) <= LOGIT_TOL
    assert rel_err(fast, ref) <= FAST_TOL
    with pytest.raises(B.StError):
        g.prefill(toks[:4], two_term=True, fast=True)      # the two flags exclude each other
    g.close()


def test_long_pass_through_64_layers_of_a_narrow_model():
    """Depth pin: a model as deep as the 32B one (64 layers) but narrow enough for the oracle (hidden 1024, 8 query /
    2 kv heads of 128, intermediate 2816, vocab 4096).  A 300-row pass, the same rows in passes of at most 256, and
    the decode step at the same position all stay within the tolerance of the oracle through the full depth, and
    the default pass (two bf16 terms, and with the fp16 weight copy attached: single fp16 operands) is no further from
    it than 1.5 times the decode step -- whose only rounding is the bf16 K/V cache -- so what error a long pass has
    is the cache's, not its own.  The opt-in single-term pass is bounded too."""
    print_case("narrow 64-layer model: 300-row pass (default, single-term, <=256-row passes) and decode at row 300")
    cfg, g, o = make_pair("qwen1p5b", 5, max_seq=340, max_chunk=320, n_layers=64, gen_device="cuda",
                          hidden=1024, n_q_heads=8, n_kv_heads=2, intermediate=2816, vocab=4096, tie_embeddings=0)
    toks = synth.make_prompt(300, cfg["vocab"], 21)
    ref = o.feed(toks)
    errs = {}
    for name, kw in (("default", {}), ("single-term", {"fast": True}), ("<=256 rows", {"two_term": True})):
        g.truncate(0)
        errs[name] = rel_err(g.prefill(toks, **kw)[0], ref)
    g.truncate(0)
    g.prefill(toks[:299], want_logits=False)
    errs["decode"] = rel_err(g.decode_step(int(toks[299]))[0], ref)
    g.attach_f16()                                        # the same pass on the fp16 MFMA with fp16 activations
    g.truncate(0)
    errs["fp16 operands"] = rel_err(g.prefill(toks)[0], ref)
    print_case(errs)
    assert max(errs["default"], errs["<=256 rows"], errs["decode"], errs["fp16 operands"]) <= LOGIT_TOL
    assert errs["default"] <= 1.5 * errs["decode"] and errs["fp16 operands"] <= 1.5 * errs["decode"]
    assert errs["single-term"] <= FAST_TOL
    g.close()


@pytest.mark.parametrize("m", [1, 21, 32, 33, 86, 128, 129, 160, 192, 193, 257, 513])
def test_f16_operand_mode_regime_boundaries(m):
    """With the fp16 weight copy attached, default passes run their O, gate/up and down GEMMs on the fp16 MFMA (single
    fp16 activations; the QKV input and the queries stay in two bf16 terms) -- in the streaming kernel up to 128 rows,
    in the ring kernel above: chunk lengths around the kernel switches, on top of 100 cached keys, against the oracle
    (2 layers); the decode step is unchanged."""
    print_case(f"1.5B shape, 2 layers, fp16 operand mode: 100 cached + chunk of {m}")
    cfg, g, o = make_pair("qwen1p5b", 11, max_seq=640, max_chunk=520, n_layers=2, gen_device="cuda")
    g.attach_f16()
    prompt = synth.make_prompt(100 + m, cfg["vocab"], 12)
    assert _teacher_forced(cfg, g, o, prompt, [100, m], 1) <= LOGIT_TOL
    g.close()


def test_f16_operand_mode_at_full_depth_and_tail_tiles():
    """fp16 operand mode through all 28 layers of the 1.5B shape (300-row pass against the oracle: within the
    tolerance and within 1.3x of the two-term pass), then detached again (bit-identical to before); and a 4096-row
    pass of the custom shape that takes every leftover-tile path of the ring GEMM, in fp16."""
    print_case("1.5B shape, 28 layers: 300-token prompt, two bf16 terms against fp16 operands")
    cfg, g, o = make_pair("qwen1p5b", 1, max_seq=320, max_chunk=300, gen_device="cuda")
    toks = synth.make_prompt(300, cfg["vocab"], 21)
    ref = o.feed(toks)
    two, _ = g.prefill(toks)
    g.attach_f16()
    g.truncate(0)
    f16, _ = g.prefill(toks)
    g.attach_f16(False)
    g.truncate(0)
    again, _ = g.prefill(toks)
    print_case("two bf16 terms", rel_err(two, ref), "fp16 operands", rel_err(f16, ref))
    assert rel_err(f16, ref) <= LOGIT_TOL and rel_err(f16, ref) <= 1.3 * rel_err(two, ref)
    assert np.array_equal(two, again) and not np.array_equal(two, f16)
    g.close()
    o.close()
    print_case("custom shape (hidden 4288, intermediate 2240): 1 layer, 40 cached + 4096-row chunk, fp16 operands")
    cfg, g, o = make_pair("qwen1p5b", 31, max_seq=4200, max_chunk=4096, n_layers=1, gen_device="cuda",
                          hidden=4288, intermediate=2240, n_q_heads=6, n_kv_heads=1, vocab=2048)
    g.attach_f16()
    prompt = synth.make_prompt(4136, cfg["vocab"], 32)
    assert _teacher_forced(cfg, g, o, prompt, [40, 4096], 2) <= LOGIT_TOL
    g.close()


def test_f16_attach_rejects_what_it_cannot_hold():
    """A weight beyond the fp16 range keeps the mode off (ST_ERANGE, passes stay in two bf16 terms); a shape whose
    intermediate size is not a multiple of 64 is refused (ST_EINVAL); a short buffer too (ST_ENOMEM)."""
    cfg = synth.model_config("qwen1p5b", max_seq=400, max_chunk=320, n_layers=1)
    w = synth.make_weights(cfg, 3, device="cuda")
    g = B.Model(cfg, w)
    toks = synth.make_prompt(300, cfg["vocab"], 4)
    before, _ = g.prefill(toks)
    w["layers"][0]["w_down"][5, 7] = 1.0e5
    with pytest.raises(B.StError) as e:
        g.attach_f16()
    assert e.value.code == B.ST_ERANGE
    w["layers"][0]["w_down"][5, 7] = 0.0
    n = B.C.c_size_t()
    B._check(B.lib().st_query_f16_bytes(B.C.byref(B.make_config(cfg)), B.C.byref(n)))
    small = torch.empty(n.value - 256, dtype=torch.uint8, device="cuda")
    assert B.lib().st_model_attach_f16(g._h, small.data_ptr(), small.numel()) == B.ST_ENOMEM
    g.truncate(0)
    after, _ = g.prefill(toks)                            # still the two-term pass (one weight differs: now 0)
    assert np.isfinite(after).all() and rel_err(after, before) < 0.05
    g.close()
    tiny = synth.model_config("tiny_small", max_seq=64, max_chunk=64)
    assert B.lib().st_query_f16_bytes(B.C.byref(B.make_config(tiny)), B.C.byref(n)) == B.ST_EINVAL
