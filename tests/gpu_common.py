"""Shared helpers of the GPU parity tests: builds a model on both sides from the same bf16 bits."""
import numpy as np
import torch

from oracle import oracle as O
from paper_2504_12329_amd import binding as B, synth

LOGIT_TOL = 2e-2     # max |gpu - oracle| / max |oracle| per logit vector, bf16 path vs fp32 oracle


def rel_err(gpu, orc):
    orc = np.asarray(orc, dtype=np.float64)
    return float(np.abs(np.asarray(gpu, dtype=np.float64) - orc).max() / np.abs(orc).max())


def make_pair(name, seed, max_seq, max_chunk=None, n_layers=None, gen_device="cpu", **over):
    """(cfg, gpu Model, OracleModel) sharing one set of bf16 weight bits."""
    cfg = synth.model_config(name, max_seq=max_seq, max_chunk=max_chunk, n_layers=n_layers)
    cfg.update(over)
    w = synth.make_weights(cfg, seed, device=gen_device)
    if not cfg["qkv_bias"]:
        for lw in w["layers"]:
            lw["bqkv"].zero_()
    orc = O.OracleModel(synth.oracle_config(cfg), synth.oracle_views(cfg, w))
    wg = dict(embed=w["embed"].cuda(), final_norm=w["final_norm"].cuda(),
              lm_head=None if w["lm_head"] is None else w["lm_head"].cuda(),
              layers=[{k: v.cuda() for k, v in lw.items()} for lw in w["layers"]])
    gpu = B.Model(cfg, wg)
    return cfg, gpu, orc


def print_case(*a):
    print(*a, flush=True)
