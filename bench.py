"""Benchmark of the Speculative Thinking hot path on one MI355X.

One "step" is one whole generation job of the speculative (1.5B-shaped) model: catch-up prefill
of a 512-token prompt onto an empty cache, 4096 chained greedy decode steps (every projection,
the split attention, LM head and arg-max), and the trigger scan over the produced tokens, all
enqueued without host round trips.  `value` is output tokens per second over the timed jobs with
weights, prompt and cache resident in HBM.  Prints one JSON line.

Besides the headline it reports, in the same line: decode throughput and HBM fraction in windows
around kv = 1k / 2k / 4k, the roofline of the kernel that moves the most bytes, the target
(32B-shaped) model's decode and catch-up prefill rates, a short run of the whole two-model loop
at the paper's hand-over density, and the CPU oracle timed on this machine.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PROMPT, N_DECODE = 512, 4096
HBM_PEAK = 8.0e12          # bytes/s, MI355X HBM3E
# HBM bytes per launch of k_gateup_swiglu<3,1,true> from rocprofv3 FETCH_SIZE (x2.00) + WRITE_SIZE (x1.00), see
# profiles/decode_qwen1p5b_hbm_counters.md; set to None whenever that kernel changes until the counters are re-taken
GATEUP_TRAFFIC_BYTES = 55.29e6
MFMA_PEAK = 2.5e15         # dense bf16 flop/s


def cpu_baseline(cfg, w_gpu, prompt):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the same workload: a 64-token
    prompt pass and 16 greedy decode steps at all cores, then 6 more decode steps on one core."""
    import ctypes
    from oracle import oracle as O
    from paper_2504_12329_amd import synth
    ocfg = synth.oracle_config(dict(cfg, max_seq=128))
    orc = O.OracleModel(ocfg, synth.oracle_views(cfg, w_gpu))
    n_pre, n_dec, n_one = 64, 16, 6
    cores = int(O.lib().orc_threads())
    t0 = time.perf_counter()
    tok = O.argmax(orc.feed(prompt[:n_pre]))
    t_pre = time.perf_counter() - t0
    t0 = time.perf_counter()
    for _ in range(n_dec):
        tok = O.argmax(orc.feed([tok]))
    t_dec = time.perf_counter() - t0
    # one core: the oracle's loops are OpenMP, so the thread count is set through the OpenMP runtime it links
    omp = ctypes.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(1)
    t0 = time.perf_counter()
    for _ in range(n_one):
        tok = O.argmax(orc.feed([tok]))
    t_one = time.perf_counter() - t0
    omp.omp_set_num_threads(cores)
    orc.close()
    return {"value": n_dec / t_dec, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "prefill_tok_s": n_pre / t_pre, "one_core": {"value": n_one / t_one, "unit": "tokens/s", "cores": 1},
            "sample": f"the same 1.5B-shaped model in fp32: {n_pre}-token prompt pass, then {n_dec} greedy decode "
                      f"steps on {cores} cores (kv length {n_pre}..{n_pre + n_dec}), then {n_one} more on one core.  "
                      "The GPU figure is quoted at kv 1k..4k; the oracle cannot reach that context inside the sample "
                      "(it would feed 1k tokens one by one), and at kv 1k its attention would add 0.5 % to the bytes "
                      "a token reads"}


def batched_decode(torch, B, synth, cost, cfg, w, n_seq=16, steps=24):
    """16 independent sequences with prompts of 128..1024 tokens (uniform, seed 4) decoding together on one model."""
    import numpy as np
    cfg = dict(cfg, max_seq=1200, max_chunk=max(64, min(cfg["max_chunk"], 1024)))
    batch = B.Batch(cfg, w, n_seq)
    lens = np.random.default_rng(4).integers(128, 1025, n_seq)
    for s in range(n_seq):
        batch.prefill(s, synth.make_prompt(int(lens[s]), cfg["vocab"], 50 + s), want_logits=False)
    seqs, toks = np.arange(n_seq, dtype=np.int32), np.ones(n_seq, np.int32)
    for _ in range(3):
        _, toks = batch.decode_step(seqs, toks)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        _, toks = batch.decode_step(seqs, toks)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    batch.close()
    return {"n_seq": n_seq, "prompt_lengths": [int(v) for v in lens], "ms_per_step": dt * 1e3, "tok_s": n_seq / dt,
            "weight_GB_s": cost.weight_bytes(cfg) / dt / 1e9, "hbm_frac": cost.weight_bytes(cfg) / dt / HBM_PEAK}


def single_decode(torch, B, synth, cost, cfg, w, kv0=4096, steps=40, single_kernel=False):
    """Greedy decode rate of one sequence at a context of about kv0 tokens (chained, captured steps); with
    single_kernel the step is the persistent kernel the library offers as an alternative (ST_DECODE_PERSIST=1)."""
    cfg = dict(cfg, max_seq=kv0 + 128, max_chunk=min(cfg["max_chunk"], 4096))
    old = os.environ.get("ST_DECODE_PERSIST")
    os.environ["ST_DECODE_PERSIST"] = "1" if single_kernel else "0"
    try:
        model = B.Model(cfg, w)
    finally:
        if old is None:
            del os.environ["ST_DECODE_PERSIST"]
        else:
            os.environ["ST_DECODE_PERSIST"] = old
    assert model.step_kind() == (1 if single_kernel else 0)
    toks = torch.from_numpy(synth.make_prompt(kv0, cfg["vocab"], 5)).cuda()
    for lo in range(0, kv0, cfg["max_chunk"]):
        model.prefill_device(toks[lo:lo + cfg["max_chunk"]])
    out = torch.empty(64, dtype=torch.int32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    model.decode_greedy(0, 8, chained=True, out_dev=out)
    e0.record()
    model.decode_greedy(0, steps, chained=True, out_dev=out)
    e1.record()
    torch.cuda.synchronize()
    sec = e0.elapsed_time(e1) / 1e3 / steps
    model.close()
    nbytes = cost.decode_bytes(cfg, kv0 + 8 + steps // 2)
    return {"tok_s": 1 / sec, "GB_s": nbytes / sec / 1e9, "hbm_frac": nbytes / sec / HBM_PEAK}


def batched_loop(B, synth, cfg_s, w_s, cfg_l, w_l, n_seq=16, n_out=210, n_seg=20, period=85, staggered=False,
                 gather=0, rule=None):
    """The two-model loop for 16 sequences at once (7B-shaped speculative, 32B-shaped target), prompts of 128..1024
    tokens (uniform, seed 4), segments of 20; hand-over every 85th speculative token, or, with rule = (keyword
    modulus, delimiter modulus), whenever a sequence's own tokens satisfy previous id % delimiter == 0 and
    id % keyword == 0."""
    import numpy as np
    small, large = B.Batch(cfg_s, w_s, n_seq), B.Batch(cfg_l, w_l, n_seq)
    small.attach_f16()      # catch-up passes on fp16 operands (the decode steps are unchanged)
    large.attach_f16()
    lens = np.random.default_rng(4).integers(128, 1025, n_seq)
    vocab = cfg_s["vocab"]
    prompts = [synth.make_prompt(int(lens[i]), vocab, 50 + i) for i in range(n_seq)]
    t0 = time.perf_counter()
    if rule is None:
        # staggered: hand-overs spread over the period, as sequences that trigger on their own content would be
        phase = [(i * period) // n_seq for i in range(n_seq)] if staggered else None
        g = B.st_generate_batch(small, large, prompts, n_out, n_seg, vocab, forced_period=period,
                                forced_phase=phase, gather=gather)
        schedule = "forced: every 85th speculative token hands over" + \
                   (" (sequence i starts its count at 85*i/16)" if staggered else " (all sequences in step)")
    else:
        g = B.st_generate_batch(small, large, prompts, n_out, n_seg, vocab, kw=synth.modulo_bitmap(vocab, rule[0]),
                                delim=synth.modulo_bitmap(vocab, rule[1]), window=2, gather=gather)
        schedule = f"rule: previous id % {rule[1]} == 0 and id % {rule[0]} == 0, evaluated per sequence"
    dt = time.perf_counter() - t0
    st = g["stats"]
    small.close()
    large.close()
    return {"tok_s": st["n_out"] / dt, "n_seq": n_seq, "n_out": st["n_out"], "n_handoffs": st["n_handoffs"],
            "modify_ratio": st["n_large"] / max(1, st["n_out"]), "seconds": dt,
            "ms_small_decode": st["ms_small_decode"], "ms_large_decode": st["ms_large_decode"],
            "ms_small_prefill": st["ms_small_prefill"], "ms_large_prefill": st["ms_large_prefill"],
            "gather": gather,
            "schedule": schedule + ", target writes 20; prompt prefill included; the ms_* figures of the two models overlap"}


def target_model_extras(torch, B, synth, cost, small, sizes=(21, 86, 256, 1024, 4096), loop=True, n_layers=None,
                        batched=True, forms=("f16", "two_term", "fast")):
    """32B-shaped target: decode rate at kv ~ 4k, catch-up prefill on a 4096-token cache, and the loop.  `forms`:
    which forms of the passes of 129 rows and more are timed (a kernel profile takes one)."""
    cfg = synth.model_config("qwen32b", max_seq=4096 + 4096 + 64, max_chunk=4096, n_layers=n_layers)
    w = synth.make_weights(cfg, 2, device="cuda")
    large = B.Model(cfg, w)
    toks = torch.from_numpy(synth.make_prompt(8192, cfg["vocab"], 5)).cuda()
    out = torch.empty(64, dtype=torch.int32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if forms[0] == "f16":
        large.attach_f16()
    large.prefill_device(toks[:4096], fast=(forms[0] == "fast"))   # the cached context, in the first form asked for
    large.attach_f16(False)
    large.decode_greedy(0, 8, chained=True, out_dev=out)
    e0.record()
    large.decode_greedy(0, 20, chained=True, out_dev=out)
    e1.record()
    torch.cuda.synchronize()
    sec = e0.elapsed_time(e1) / 1e3 / 20
    res = {"decode_kv4096": {"tok_s": 1 / sec, "GB_s": cost.decode_bytes(cfg, 4110) / sec / 1e9,
                             "hbm_frac": cost.decode_bytes(cfg, 4110) / sec / HBM_PEAK}, "prefill_on_kv4096": {}}
    def timed_pass(m, fast):
        for _ in range(2):
            large.truncate(4096)
            e0.record()
            large.prefill_device(toks[4096:4096 + m], fast=fast)
            e1.record()
            torch.cuda.synchronize()
        sec = e0.elapsed_time(e1) / 1e3
        fl = cost.prefill_flops(cfg, m, 4096)
        return {"ms": sec * 1e3, "tok_s": m / sec, "TFLOP_s": fl / sec / 1e12, "mfma_frac": fl / sec / MFMA_PEAK,
                "weight_GB_s": cost.weight_bytes(cfg) / sec / 1e9, "hbm_frac": cost.weight_bytes(cfg) / sec / HBM_PEAK,
                "bound": "hbm" if m < 312 else "mfma"}

    # Forms of a pass.  The headline entry of every size is the default-precision pass of a model that has been
    # given the fp16 copy of its projection weights (st_model_attach_f16: fp16 MFMA, single fp16 activations);
    # "two_term_bf16" is the same precision without that copy (two bf16 terms: twice the MFMA work, which is free
    # while the weight stream sets the time); "fast_single_term" (129 rows and more) is ST_PREFILL_FAST (single bf16
    # inputs, about twice the logit error).  The first two meet the logit tolerance against the oracle at every depth
    # tested.
    side = {}
    for m in sizes:
        side[m] = {}
        if "two_term" in forms:
            side[m]["two_term_bf16"] = timed_pass(m, False)
        if m > 128 and "fast" in forms:
            side[m]["fast_single_term"] = timed_pass(m, True)
    if "f16" in forms:
        large.attach_f16()
        for m in sizes:
            res["prefill_on_kv4096"][str(m)] = dict(timed_pass(m, False), form="fp16 operands", **side[m])
        large.attach_f16(False)
    else:
        for m in sizes:
            res["prefill_on_kv4096"][str(m)] = side[m]
    large.close()
    del large
    if not batched:
        return res
    res["batched_decode"] = {"qwen32b": batched_decode(torch, B, synth, cost, cfg, w)}
    if loop:
        cfg7 = synth.model_config("qwen7b", max_seq=2100, max_chunk=4096)
        w7 = synth.make_weights(cfg7, 4, device="cuda")
        res["decode_7b_kv4096"] = single_decode(torch, B, synth, cost, cfg7, w7)
        res["batched_decode"]["qwen7b"] = batched_decode(torch, B, synth, cost, cfg7, w7)
        cfg_l = dict(cfg, max_seq=2100, max_chunk=4096)
        res["loop_batched_7b_32b"] = batched_loop(B, synth, cfg7, w7, cfg_l, w)
        # the configured workload closer to its stated length: 1000 outputs per sequence under the trigger rule itself
        # (fires about once in 8600 uniform ids) and under a rule of the paper's trigger density (once in 105);
        # the hand-overs realised on the models' own greedy output are reported
        res["loop_batched_7b_32b_rule"] = batched_loop(B, synth, cfg7, w7, cfg_l, w, n_out=1000, rule=(97, 89))
        res["loop_batched_7b_32b_rule_dense"] = batched_loop(B, synth, cfg7, w7, cfg_l, w, n_out=1000, rule=(15, 7),
                                                             gather=4)
        # the same job with the hand-overs spread over the period: target passes held until all sequences wait
        # (gather = n_seq), and started at once (gather = 0), which leaves the target with one or two rows per pass
        res["loop_batched_7b_32b_staggered"] = batched_loop(B, synth, cfg7, w7, cfg_l, w, staggered=True, gather=16)
        res["loop_batched_7b_32b_staggered"]["tok_s_without_gather"] = batched_loop(
            B, synth, cfg7, w7, cfg_l, w, staggered=True, gather=0)["tok_s"]
        del w7
    # the whole two-model loop at the paper's density: hand-over every 85 speculative tokens, segments of 20
    # (both models must share one vocabulary: the target is re-wrapped over the first 151936 rows of its
    # embedding and LM head, the speculative model's vocabulary size)
    if not loop:
        return res
    vocab = small.cfg["vocab"]
    cfg_l = dict(cfg, vocab=vocab, max_seq=5376, max_chunk=256)
    w_l = dict(w, embed=w["embed"][:vocab], lm_head=w["lm_head"][:vocab])
    large = B.Model(cfg_l, w_l)
    large.attach_f16()      # catch-up passes on fp16 operands (the speculative model got its copy in main())
    small.truncate(0)
    prompt = synth.make_prompt(256, vocab, 7)
    n_out = 1050
    t0 = time.perf_counter()
    g = B.st_generate(small, large, None, prompt, n_out, 20, forced_period=85)
    dt = time.perf_counter() - t0
    st = g["stats"]
    res["loop_1p5b_32b"] = {"tok_s": st["n_out"] / dt, "n_out": st["n_out"], "n_handoffs": st["n_handoffs"],
                            "modify_ratio": st["n_large"] / max(1, st["n_out"]),
                            "ms_small_decode": st["ms_small_decode"], "ms_large_decode": st["ms_large_decode"],
                            "ms_small_prefill": st["ms_small_prefill"], "ms_large_prefill": st["ms_large_prefill"],
                            "schedule": "forced: every 85th speculative token hands over, target writes 20"}
    # the same pair under the synthetic trigger rule itself (previous id % 89 == 0 and id % 97 == 0), 5000 output
    # tokens: on uniform ids the rule fires about once in 8600 tokens, so a run has zero or one hand-over and is in
    # effect the speculative model's decode rate; the realised hand-overs and their catch-up lengths are reported
    small.truncate(0)
    large.truncate(0)
    rule = B.TriggerRule(vocab, synth.modulo_bitmap(vocab, 97), synth.modulo_bitmap(vocab, 89), 2)
    cfg_s = small.cfg
    if cfg_s["max_seq"] >= 256 + 5000:
        t0 = time.perf_counter()
        g = B.st_generate(small, large, rule, prompt, 5000, 20)
        dt = time.perf_counter() - t0
        st = g["stats"]
        res["loop_1p5b_32b_rule"] = {
            "tok_s": st["n_out"] / dt, "n_out": st["n_out"], "n_handoffs": st["n_handoffs"],
            "target_catch_up_lengths": [sp["large_prefill_hi"] - sp["large_prefill_lo"] for sp in g["spans"]],
            "ms_small_decode": st["ms_small_decode"], "ms_large_decode": st["ms_large_decode"],
            "ms_small_prefill": st["ms_small_prefill"], "ms_large_prefill": st["ms_large_prefill"],
            "schedule": "rule: previous id % 89 == 0 and id % 97 == 0, target writes 20"}
    # and under a rule of the paper's trigger density (previous id % 7 == 0 and id % 15 == 0: about one token in 105
    # on uniform ids, Section 3 (1)); the density realised on this model's own greedy output is reported
    small.truncate(0)
    large.truncate(0)
    rule = B.TriggerRule(vocab, synth.modulo_bitmap(vocab, 15), synth.modulo_bitmap(vocab, 7), 2)
    t0 = time.perf_counter()
    g = B.st_generate(small, large, rule, prompt, 1500, 20)
    dt = time.perf_counter() - t0
    st = g["stats"]
    res["loop_1p5b_32b_rule_dense"] = {
        "tok_s": st["n_out"] / dt, "n_out": st["n_out"], "n_handoffs": st["n_handoffs"],
        "modify_ratio": st["n_large"] / max(1, st["n_out"]),
        "target_catch_up_lengths": [sp["large_prefill_hi"] - sp["large_prefill_lo"] for sp in g["spans"]],
        "ms_small_decode": st["ms_small_decode"], "ms_large_decode": st["ms_large_decode"],
        "ms_small_prefill": st["ms_small_prefill"], "ms_large_prefill": st["ms_large_prefill"],
        "schedule": "rule: previous id % 7 == 0 and id % 15 == 0, target writes 20"}
    # the non-reasoning-speculator schedule (Section 4.3): the target writes the first 100 tokens and takes over for
    # 20 tokens after every delimiter; the delimiter class id % 24 == 0 would give a modify ratio near 44 % on
    # uniform tokens, the realised ratio is reported
    small.truncate(0)
    large.truncate(0)
    t0 = time.perf_counter()
    g = B.st_generate_policy(small, large, prompt, 600, vocab, delim=B.host_bitmap(vocab, range(0, vocab, 24)),
                             sentence_len=1, unconditional=True, n1=20, initial_target=100)
    dt = time.perf_counter() - t0
    st = g["stats"]
    res["loop_nonreasoning_1p5b_32b"] = {
        "tok_s": st["n_out"] / dt, "n_out": st["n_out"], "n_takeovers": st["n_handoffs"],
        "modify_ratio": st["n_large"] / max(1, st["n_out"]),
        "ms_small_decode": st["ms_small_decode"], "ms_large_decode": st["ms_large_decode"],
        "ms_small_prefill": st["ms_small_prefill"], "ms_large_prefill": st["ms_large_prefill"],
        "schedule": "target writes the first 100 tokens, then 20 tokens after every delimiter (id % 24 == 0)"}
    large.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--decode-steps", type=int, default=N_DECODE, help="decode steps per job (shorten for profiling)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the 32B-shaped model and the two-model loop")
    ap.add_argument("--prefill-sizes", default="21,86,256,1024,4096",
                    help="catch-up chunk lengths timed on the 32B-shaped model (one size for a kernel profile)")
    ap.add_argument("--prefill-forms", default="f16,two_term,fast",
                    help="profiling aid: forms of the long passes to time (f16, two_term, fast); the first also fills the cache")
    ap.add_argument("--extras-layers", type=int, default=None,
                    help="profiling aid: give the 32B-shaped model this many layers (per-kernel figures are unchanged)")
    ap.add_argument("--prefill-only", action="store_true",
                    help="profiling aid: with --only-extras, stop after the 32B-shaped decode / catch-up timings")
    ap.add_argument("--only-extras", action="store_true",
                    help="profiling aid: run only the 32B-shaped decode / prefill measurements, no headline job")
    ap.add_argument("--no-roofline", action="store_true",
                    help="skip the decode windows and the per-launch event timing (for counter-collection runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this path uses no second GPU, run with --gpus 1")

    import numpy as np
    import torch
    from paper_2504_12329_amd import binding as B, cost, synth

    torch.cuda.set_device(0)
    sizes = tuple(int(v) for v in args.prefill_sizes.split(","))
    if args.only_extras:
        print(json.dumps({"target_model_32b": target_model_extras(torch, B, synth, cost, None, sizes, loop=False,
                                                                       n_layers=args.extras_layers,
                                                                       batched=not args.prefill_only,
                                                                       forms=tuple(args.prefill_forms.split(",")))}))
        return
    n_dec = args.decode_steps
    cfg = synth.model_config("qwen1p5b", max_seq=max(PROMPT + N_DECODE + 64, 256 + 5000 + 64), max_chunk=PROMPT)
    w = synth.make_weights(cfg, 1, device="cuda")
    model = B.Model(cfg, w)
    model.attach_f16()      # the prompt pass runs on fp16 operands (default precision); decode is unaffected
    prompt = synth.make_prompt(PROMPT, cfg["vocab"], 3)
    prompt_dev = torch.from_numpy(prompt).cuda()
    out_dev = torch.empty(N_DECODE, dtype=torch.int32, device="cuda")
    rule = B.TriggerRule(cfg["vocab"], synth.modulo_bitmap(cfg["vocab"], 97), synth.modulo_bitmap(cfg["vocab"], 89), 2)
    hits_dev = torch.empty(65, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    def job():
        model.truncate(0)
        model.prefill_device(prompt_dev)                  # one 512-row pass, default precision
        model.decode_greedy(0, n_dec, chained=True, out_dev=out_dev)
        B._check(B.lib().st_trigger_scan(ctypes.byref(rule.c), out_dev.data_ptr(), 0, n_dec, hits_dev[1:].data_ptr(),
                                         64, hits_dev.data_ptr(), None, stream, B.ST_OUT_DEVICE))

    for _ in range(args.warmup):
        job()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        job()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = args.steps * n_dec / dt

    # decode-only windows of 128 steps centred on kv = 1024 / 2048 / 4096
    windows = {}
    model.truncate(0)
    model.prefill_device(prompt_dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for kv in (1024, 2048, 4096):
        if args.no_roofline or kv + 64 > PROMPT + n_dec:
            break
        lead = kv - 64 - model.kv_len
        model.decode_greedy(0, lead, chained=True, out_dev=out_dev)
        e0.record()
        model.decode_greedy(0, 128, chained=True, out_dev=out_dev)
        e1.record()
        torch.cuda.synchronize()
        sec = e0.elapsed_time(e1) / 1e3 / 128
        windows[str(kv)] = {"tok_s": 1.0 / sec, "GB_s": cost.decode_bytes(cfg, kv) / sec / 1e9,
                            "hbm_frac": cost.decode_bytes(cfg, kv) / sec / HBM_PEAK}

    # roofline of the kernel that moves the most bytes (gate/up projection): HIP events on every launch,
    # recorded inside the library on the stream the kernel runs on
    model.truncate(min(2048, model.kv_len))
    gu, st = [], []
    for _ in range(10 if args.no_roofline else 40):
        a, b = model.decode_step_timed()
        gu.append(a)
        st.append(b)
    gu_us = float(np.mean(gu[8:]))
    bytes_per_launch = 2 * cfg["intermediate"] * cfg["hidden"] * 2
    achieved = bytes_per_launch / (gu_us * 1e-6)
    # the whole decode step first (all kernels of a token: algorithmic bytes of the token over the step time in the
    # kv window where it is lowest), then the kernel that moves the most bytes
    worst = min(windows, key=lambda k: windows[k]["hbm_frac"]) if windows else None
    whole = None if worst is None else {
        "bound": "hbm", "scope": f"whole decode step, 128-step window at kv {worst}",
        "achieved": windows[worst]["GB_s"], "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": windows[worst]["hbm_frac"]}
    roofline = {"whole_step": whole,
                "bound": "hbm", "kernel": "k_gateup_swiglu", "achieved": achieved / 1e9, "peak": HBM_PEAK / 1e9,
                "unit": "GB/s", "frac": achieved / HBM_PEAK, "traffic": GATEUP_TRAFFIC_BYTES,
                "bytes_per_launch": bytes_per_launch, "avg_launch_us": gu_us,
                "launches_timed": len(gu[8:]) * cfg["n_layers"]}

    line = {
        "metric": "decode tok/s + HBM GB/s fraction (1.5B, 32B); handoff prefill tok/s + MFMA util",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "qwen2.5-1.5B-shaped greedy decode: 512-token random prompt prefill + 4096 decode "
                               "steps + trigger scan, batch 1, contiguous bf16 KV cache, seeded random bf16 weights",
                   "prompt_tokens": PROMPT, "decode_steps": n_dec,
                   "prefill_operands": "fp16 MFMA on an fp16 copy of the bf16 projection weights (st_model_attach_f16)"},
        "decode_windows": windows,
        "whole_step_us_ungraphed": float(np.mean(st[8:])),
        # the same step as one persistent kernel (opt-in alternative), beside the default at the same context
        "single_kernel_step_kv4096": {"single_kernel": single_decode(torch, B, synth, cost, cfg, w, single_kernel=True),
                                      "kernel_per_stage": single_decode(torch, B, synth, cost, cfg, w)},
        "algorithmic_bytes_per_token": {k: cost.decode_bytes(cfg, int(k)) for k in windows},
        "roofline": roofline,
    }
    if not args.no_extras:
        line["target_model_32b"] = target_model_extras(torch, B, synth, cost, model, sizes)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg, w, prompt)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
