"""Where the time of the persistent single-kernel decode step goes: per-stage timestamps of three blocks.

Usage:  python -m paper_2504_12329_amd.persist_stages [shape] [kv] [layers]     (build first:
        python -c "from paper_2504_12329_amd import build; build.build(); build.build_stage_profiling()")

Loads _build/libst_prof.so (the library compiled with -DST_PERSIST_PROF: thread 0 of blocks 0, 101 and the last one
stores the 100 MHz wall clock after every stage of every layer), runs chained decode steps of a seeded random model of
the given shape at a context of kv tokens, and prints the mean time per stage over the layers of the last step.
"""
import ctypes as C
import os
import sys

import numpy as np
import torch

from . import binding as B, build, synth


def main(name="qwen1p5b", kv=2048, layers=None):
    os.environ["ST_DECODE_PERSIST"] = "1"
    B.LIB_PATH = os.path.join(build.OBJ, "libst_prof.so")
    cfg = synth.model_config(name, max_seq=kv + 256, max_chunk=512, n_layers=layers)
    w = synth.make_weights(cfg, 1, device="cuda")
    m = B.Model(cfg, w)
    assert m.step_kind() == 1, "the shape does not fit the single-kernel step"
    prompt = torch.from_numpy(synth.make_prompt(512, cfg["vocab"], 3)).cuda()
    done = 0
    while done < kv:
        n = min(512, kv - done)
        m.prefill_device(prompt[:n])
        done += n
    out = torch.empty(256, dtype=torch.int32, device="cuda")
    m.decode_greedy(0, 32, chained=True, out_dev=out)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    m.decode_greedy(0, 64, chained=True, out_dev=out)
    e1.record()
    torch.cuda.synchronize()
    print(f"{name}, context {kv + 96}: {e0.elapsed_time(e1) * 1e3 / 64:.1f} us per step (with the timestamps compiled in)")
    buf = (C.c_ulonglong * (3 * 4096))()
    rc = B.lib().st_debug_persist_prof(buf)
    assert rc == 0, rc
    stamps = np.array(buf[:], dtype=np.int64).reshape(3, 4096)
    nl, nkv, nq = cfg["n_layers"], cfg["n_kv_heads"], cfg["n_q_heads"]
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    # the kernel's own split of the context into key ranges, and the work items of the range merge
    s_cap = min(128, n_cu // nkv)
    t_keys = kv + 96
    chunk = -(-(-(-t_keys // s_cap)) // 64) * 64
    s_act = -(-t_keys // chunk)
    dsl = 4
    while dsl < cfg["head_dim"] and nq * (cfg["head_dim"] // dsl) > n_cu:
        dsl *= 2
    items = nq * (cfg["head_dim"] // dsl)
    base = ["wait x", "norm", "QKV (loads held)", "QKV (streamed)", "QKV out", "ATTN", "MERGE", "wait attention",
            "O (held)", "O (streamed)", "O out", "wait x'", "norm", "gate/up (held)", "gate/up (streamed)", "SwiGLU out",
            "wait SwiGLU", "down (held)", "down (streamed)", "down out"]
    for slot, bid in enumerate((0, 101, n_cu - 1)):
        names = []
        for n in base:
            if n == "ATTN":
                names += ["wait q", "rotate", "tiles", "reduce + out"] if bid < s_act * nkv else ["(no key range)"]
            elif n == "MERGE":
                names += ["wait ranges", "merge"] if (s_act > 1 and bid < items) else ["(no merge item)"]
            else:
                names.append(n)
        per = len(names) + 1
        if per * nl > 4096:
            print("too many layers for the timestamp buffer")
            return
        t = stamps[slot, : per * nl].reshape(nl, per)
        us = np.diff(t, axis=1)[min(2, nl - 1):].mean(axis=0) / 100.0
        print(f"block {bid}: {(t[min(2, nl - 1):, -1] - t[min(2, nl - 1):, 0]).mean() / 100.0:.2f} us per layer")
        for n, v in zip(names, us):
            print(f"    {n:22s} {v:6.2f}")
    m.close()


if __name__ == "__main__":
    a = sys.argv[1:]
    main(a[0] if a else "qwen1p5b", int(a[1]) if len(a) > 1 else 2048, int(a[2]) if len(a) > 2 else None)
