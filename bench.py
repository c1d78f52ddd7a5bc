"""Benchmark of the Speculative Thinking hot path on one MI355X.

One "step" is one whole generation job of the speculative (1.5B-shaped) model: catch-up prefill
of a 512-token prompt onto an empty cache, 4096 chained greedy decode steps (every projection,
the split attention, LM head and arg-max), and the trigger scan over the produced tokens, all
enqueued without host round trips.  `value` is output tokens per second over the timed jobs with
weights, prompt and cache resident in HBM.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PROMPT, N_DECODE = 512, 4096
HBM_PEAK = 8.0e12          # bytes/s, MI355X HBM3E


def cpu_baseline(cfg, w_gpu, prompt):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the same workload."""
    import numpy as np
    from oracle import oracle as O
    from paper_2504_12329_amd import synth
    ocfg = synth.oracle_config(dict(cfg, max_seq=64))
    orc = O.OracleModel(ocfg, synth.oracle_views(cfg, w_gpu))
    n_pre, n_dec = 8, 24
    lg = orc.feed(prompt[:n_pre])
    tok = O.argmax(lg)
    t0 = time.perf_counter()
    for _ in range(n_dec):
        tok = O.argmax(orc.feed([tok]))
    dt = time.perf_counter() - t0
    cores = O.lib().orc_threads()
    orc.close()
    return {"value": n_dec / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n_dec} greedy decode steps of the same 1.5B-shaped model after an {n_pre}-token prompt "
                      f"(kv length {n_pre}..{n_pre + n_dec}), fp32 weights"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this path uses no second GPU, run with --gpus 1")

    import numpy as np
    import torch
    from paper_2504_12329_amd import binding as B, cost, synth

    torch.cuda.set_device(0)
    cfg = synth.model_config("qwen1p5b", max_seq=PROMPT + N_DECODE + 64, max_chunk=PROMPT)
    w = synth.make_weights(cfg, 1, device="cuda")
    model = B.Model(cfg, w)
    prompt = synth.make_prompt(PROMPT, cfg["vocab"], 3)
    prompt_dev = torch.from_numpy(prompt).cuda()
    out_dev = torch.empty(N_DECODE, dtype=torch.int32, device="cuda")
    rule = B.TriggerRule(cfg["vocab"], synth.modulo_bitmap(cfg["vocab"], 97), synth.modulo_bitmap(cfg["vocab"], 89), 2)
    hits_dev = torch.empty(65, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    def job():
        model.truncate(0)
        model.prefill_device(prompt_dev)
        model.decode_greedy(0, N_DECODE, chained=True, out_dev=out_dev)
        B._check(B.lib().st_trigger_scan(__import__("ctypes").byref(rule.c), out_dev.data_ptr(), 0, N_DECODE,
                                         hits_dev[1:].data_ptr(), 64, hits_dev.data_ptr(), None, stream,
                                         B.ST_OUT_DEVICE))

    for _ in range(args.warmup):
        job()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        job()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = args.steps * N_DECODE / dt

    # decode-only windows of 128 steps centred on kv = 1024 / 2048 / 4096
    windows = {}
    model.truncate(0)
    model.prefill_device(prompt_dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for kv in (1024, 2048, 4096):
        lead = kv - 64 - model.kv_len
        model.decode_greedy(0, lead, chained=True, out_dev=out_dev)
        e0.record()
        model.decode_greedy(0, 128, chained=True, out_dev=out_dev)
        e1.record()
        torch.cuda.synchronize()
        sec = e0.elapsed_time(e1) / 1e3 / 128
        windows[str(kv)] = {"tok_s": 1.0 / sec, "GB_s": cost.decode_bytes(cfg, kv) / sec / 1e9,
                            "hbm_frac": cost.decode_bytes(cfg, kv) / sec / HBM_PEAK}

    # roofline of the dominant kernel (gate/up projection): per-launch HIP events inside the library
    model.truncate(2048)
    gu, st = [], []
    for _ in range(40):
        a, b = model.decode_step_timed()
        gu.append(a)
        st.append(b)
    gu_us = float(np.mean(gu[8:]))
    bytes_per_launch = 2 * cfg["intermediate"] * cfg["hidden"] * 2
    achieved = bytes_per_launch / (gu_us * 1e-6)
    roofline = {"bound": "hbm", "kernel": "k_gateup_swiglu", "achieved": achieved / 1e9, "peak": HBM_PEAK / 1e9,
                "unit": "GB/s", "frac": achieved / HBM_PEAK, "traffic": None,
                "bytes_per_launch": bytes_per_launch, "avg_launch_us": gu_us,
                "launches_timed": len(gu[8:]) * cfg["n_layers"]}

    line = {
        "metric": "decode tok/s + HBM GB/s fraction (1.5B, 32B); handoff prefill tok/s + MFMA util",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "qwen2.5-1.5B-shaped greedy decode: 512-token random prompt prefill + 4096 decode "
                               "steps + trigger scan, batch 1, contiguous bf16 KV cache, seeded random bf16 weights",
                   "prompt_tokens": PROMPT, "decode_steps": N_DECODE},
        "decode_windows": windows,
        "whole_step_us_at_kv2048": float(np.mean(st[8:])),
        "algorithmic_bytes_per_token": {k: cost.decode_bytes(cfg, int(k)) for k in windows},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(cfg, w, prompt)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
