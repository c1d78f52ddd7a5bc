"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and rejects bad
arguments before touching the GPU.  No compute calls."""
import ctypes as C
import os
import re

import pytest

from paper_2504_12329_amd import binding as B, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(B.LIB_PATH):
        from paper_2504_12329_amd import build
        build.build()
    return B.lib()


def _declared():
    text = open(os.path.join(ROOT, "include", "st.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(st_[a-z0-9_]+)\s*\(", text)))


def test_exports_every_declared_symbol(L):
    names = _declared()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_struct_sizes_match_header():
    assert C.sizeof(B.st_config) == 13 * 4
    assert C.sizeof(B.st_spans) == 6 * 4
    assert C.sizeof(B.st_trigger_rule) == 2 * 8 + 2 * 4
    assert C.sizeof(B.st_gen_stats) == 4 * 4 + 4 * 8
    assert C.sizeof(B.st_policy) == 4 * 8 + 6 * 4 + 8 + 4 * 4     # 4 bitmaps, 6 ints, aux pointer, 4 ints
    assert C.sizeof(B.st_action) == 6 * 4


def test_query_sizes_and_config_validation(L):
    cfg = synth.model_config("tiny_small", 128)
    kv, ws = B.st_query_sizes(cfg)
    assert kv == 2 * 2 * 2 * 128 * 64 * 2 and ws > 0
    big = synth.model_config("qwen32b", 8192 + 64, max_chunk=4096)
    kv, ws = B.st_query_sizes(big)
    assert kv == 262144 * (8192 + 64) and ws < 2 << 30
    for key, val in [("head_dim", 96), ("hidden", 260), ("n_kv_heads", 3), ("n_layers", 0), ("max_seq", 0),
                     ("hidden", 16384), ("tie_embeddings", 2), ("rope_theta", 0.0), ("max_chunk", 0)]:
        bad = dict(cfg, **{key: val})
        with pytest.raises(B.StError) as e:
            B.st_query_sizes(bad)
        assert e.value.code == B.ST_EINVAL and str(e.value)
    with pytest.raises(B.StError):
        B.st_query_sizes(dict(cfg, n_q_heads=18, n_kv_heads=2))      # 9 query heads per kv head


def test_null_and_bad_arguments_are_rejected_before_any_launch(L):
    n = C.c_int32()
    assert L.st_kv_len(None, C.byref(n)) == B.ST_EINVAL
    assert L.st_kv_truncate(None, 0) == B.ST_EINVAL
    assert L.st_prefill(None, None, 1, None, None, 0) == B.ST_EINVAL
    assert L.st_decode_step(None, 0, None, None, 0) == B.ST_EINVAL
    assert L.st_decode_greedy(None, 0, 1, None, 0) == B.ST_EINVAL
    assert L.st_handoff(None, None, None, None, 1, 1, None, None, None, 0) == B.ST_EINVAL
    assert L.st_generate(None, None, None, 0, None, 1, 1, 1, None, None, None, 0, None) == B.ST_EINVAL
    assert b"NULL" in L.st_last_error()
    cfg = B.make_config(synth.model_config("tiny_small", 128))
    h = C.c_void_p()
    assert L.st_model_create(C.byref(cfg), None, None, 0, None, 0, None, C.byref(h)) == B.ST_EINVAL
    assert L.st_model_create(C.byref(cfg), None, None, 0, None, 0, None, None) == B.ST_EINVAL
    # trigger scan argument checks
    rule = B.st_trigger_rule(0x1000, 0, 2, 1024)
    assert L.st_trigger_scan(C.byref(rule), 0x1000, 0, 4, None, 0, C.byref(n), None, None, 0) == B.ST_EINVAL  # no delim
    rule = B.st_trigger_rule(0x1000, 0, 3, 1024)
    assert L.st_trigger_scan(C.byref(rule), 0x1000, 0, 4, None, 0, C.byref(n), None, None, 0) == B.ST_EINVAL
    rule = B.st_trigger_rule(0x1000, 0, 1, 1024)
    assert L.st_trigger_scan(C.byref(rule), 0x1000, 5, 4, None, 0, C.byref(n), None, None, B.ST_OUT_DEVICE) == B.ST_ERANGE
    assert L.st_trigger_scan(C.byref(rule), 0x1000, 0, 4, None, 0, C.byref(n), None, None, 0) == B.ST_EINVAL  # no scratch


def test_model_create_checks_buffers(L):
    cfg_d = synth.model_config("tiny_small", 128)
    cfg = B.make_config(cfg_d)
    kv, ws = B.st_query_sizes(cfg_d)
    Lyr = cfg_d["n_layers"]
    fake = (C.c_void_p * Lyr)(*([0x10000] * Lyr))
    arr = C.cast(fake, C.POINTER(C.c_void_p))
    w = B.st_weights(0x10000, 0x10000, 0x10000, arr, arr, arr, arr, arr, arr, arr)
    h = C.c_void_p()
    assert L.st_model_create(C.byref(cfg), C.byref(w), 0x10000, kv - 1, 0x20000, ws, None, C.byref(h)) == B.ST_ENOMEM
    assert L.st_model_create(C.byref(cfg), C.byref(w), 0x10000, kv, 0x20000, ws - 1, None, C.byref(h)) == B.ST_ENOMEM
    assert L.st_model_create(C.byref(cfg), C.byref(w), 0x10010, kv, 0x20000, ws, None, C.byref(h)) == B.ST_EINVAL
    holes = (C.c_void_p * Lyr)(*([0x10000] * (Lyr - 1) + [None]))
    w2 = B.st_weights(0x10000, 0x10000, 0x10000, arr, arr, C.cast(holes, C.POINTER(C.c_void_p)), arr, arr, arr, arr)
    assert L.st_model_create(C.byref(cfg), C.byref(w2), 0x10000, kv, 0x20000, ws, None, C.byref(h)) == B.ST_EINVAL
    assert b"layer" in L.st_last_error()
    w3 = B.st_weights(0x10000, 0, 0x10000, arr, arr, arr, arr, arr, arr, arr)     # untied model without lm_head
    assert L.st_model_create(C.byref(cfg), C.byref(w3), 0x10000, kv, 0x20000, ws, None, C.byref(h)) == B.ST_EINVAL
    assert not h.value


def test_long_chunk_launch_plan_covers_every_tile_once(L):
    """The block numbering of the long-chunk GEMMs (K slices, leftover column tiles cut into slices of their own,
    half-width tiles of the fused gate/up form) walked on the host for every model shape and a spread of chunk
    lengths: each output tile and K step computed by exactly one block, partial sums inside the workspace."""
    from paper_2504_12329_amd import synth
    seen_two_launches = seen_tail = False
    for name in synth.SHAPES:
        cfg = synth.model_config(name, max_seq=8448, max_chunk=8192)
        h, I = cfg["hidden"], cfg["intermediate"]
        for rows in (193, 200, 256, 257, 300, 511, 512, 513, 1000, 1024, 2047, 2048, 3000, 4095, 4096, 5000, 8192):
            launches, blocks = B.st_prefill_plan_check(cfg, rows)
            my = (rows + 255) // 256
            qd = cfg["n_q_heads"] * cfg["head_dim"]
            planned = [k % 64 == 0 for k in (h, qd, h, I)]            # QKV, O, gate/up, down: K a multiple of 64
            tiles = my * (planned[1] * ((h + 255) // 256) + planned[2] * ((I + 127) // 128))
            assert launches >= sum(planned) and blocks >= tiles
            seen_two_launches |= launches > sum(planned)
    # ragged widths: a last column tile narrower than a tile in every projection
    cfg = synth.model_config("qwen1p5b", max_seq=4200, max_chunk=4096)
    cfg.update(hidden=4288, intermediate=2240, n_q_heads=6, n_kv_heads=1)
    for rows in (257, 1024, 4000, 4096):
        launches, blocks = B.st_prefill_plan_check(cfg, rows)
        seen_tail |= rows == 4096 and launches == 5
    assert seen_two_launches and seen_tail
    assert B.st_prefill_plan_check(cfg, 192) == (0, 0) and B.st_prefill_plan_check(cfg, 1) == (0, 0)
    with pytest.raises(B.StError):
        B.st_prefill_plan_check(cfg, 4097)
    with pytest.raises(B.StError):
        B.st_prefill_plan_check(cfg, 0)


def test_long_chunk_launch_plan_on_random_shapes(L):
    """The same walk over seeded random configurations: odd widths, every group size, chunk limits from 300 to 8192."""
    import random
    from paper_2504_12329_amd import synth
    rng = random.Random(5)
    for _ in range(150):
        d, nkv, grp = rng.choice([64, 128]), rng.choice([1, 2, 4, 8]), rng.choice([1, 2, 4, 5, 6, 7, 8])
        mc = rng.choice([300, 512, 1000, 2048, 4096, 8192])
        cfg = synth.model_config("qwen1p5b", max_seq=mc + 64, max_chunk=mc)
        cfg.update(hidden=64 * rng.randint(2, 128), intermediate=8 * rng.randint(16, 3599), n_q_heads=nkv * grp,
                   n_kv_heads=nkv, head_dim=d, vocab=1024, tie_embeddings=0)
        for rows in {193, 257, mc, rng.randint(193, mc)}:
            B.st_prefill_plan_check(cfg, rows)   # raises StError naming the projection if a plan is inconsistent


def test_bench_refuses_more_than_one_gpu():
    """The path is a single-GPU one: the benchmark says so instead of starting ranks."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr


def test_single_kernel_decode_plan_on_the_host(L):
    """st_decode_persist_plan for every model shape on 256 compute units: the block's LDS request is above half and
    within all of a compute unit's 160 KB, the seven hand-over regions ascend without overlap and hold what their
    stage writes, rows are cut into 1, 2, 4 or 8 parts (few long rows into several: the down projection of the 1.5B
    shape has 6 rows of 8960 per block), and shapes the step cannot take are refused."""
    from paper_2504_12329_amd import synth
    for name in synth.SHAPES:
        cfg = synth.model_config(name, max_seq=4096, max_chunk=512)
        p = B.st_decode_persist_plan(cfg, 256)
        assert 80 * 1024 < p["lds_bytes"] <= 160 * 1024, (name, p)
        r = p["regions"] + [p["handover_words"]]
        h, d, nq, nkv = cfg["hidden"], cfg["head_dim"], cfg["n_q_heads"], cfg["n_kv_heads"]
        ranges = min(128, 256 // nkv)
        need = [h, (nq + 2 * nkv) * d, nq * ranges * (d + 2), nq * d, h, cfg["intermediate"], 2 * 256]
        for i in range(7):
            assert r[i + 1] - r[i] >= need[i], (name, i, r, need)
        assert all(q in (1, 2, 4, 8) for q in p["parts"]), p
    p = B.st_decode_persist_plan(synth.model_config("qwen1p5b", max_seq=4096, max_chunk=512), 256)
    assert p["parts"][0] == 1 and p["parts"][3] > 1        # QKV: 8 rows of 1536; down: 6 rows of 8960
    small = synth.model_config("tiny_small", max_seq=256, max_chunk=64)
    with pytest.raises(B.StError):
        B.st_decode_persist_plan(dict(small, hidden=64, n_q_heads=1, n_kv_heads=1), 256)   # rows of 64 elements
    with pytest.raises(B.StError):
        B.st_decode_persist_plan(small, 4)                 # fewer than 8 compute units
    with pytest.raises(B.StError):
        B.st_decode_persist_plan(dict(small, n_q_heads=16, n_kv_heads=16, hidden=1024), 8)  # 16 kv heads on 8 units
