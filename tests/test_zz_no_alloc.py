"""The trigger scan for callers that cannot allocate device memory (st_trigger_scan_static: staging in a static
device array inside the library) against st_trigger_scan on the same inputs, through the C ABI: two calls in a row,
the second on a smaller input, so that nothing of the first call's staging contents may leak into the second."""
import numpy as np
import pytest
import torch

from paper_2504_12329_amd import binding as B, synth

pytestmark = pytest.mark.gpu


def _tokens(rng, n, V):
    toks = rng.integers(0, V, n).astype(np.int32)
    idx = rng.integers(1, n, max(4, n // 20))
    toks[idx] = 97 * rng.integers(0, V // 97, idx.size)          # keywords ...
    toks[idx - 1] = 89 * rng.integers(0, V // 89, idx.size)      # ... right after delimiters
    return toks


@pytest.mark.parametrize("window", [1, 2, 5])
def test_static_scan_matches_the_scan_with_caller_scratch(window):
    print(f"static trigger scan, window {window}: 5000 tokens then 300 tokens", flush=True)
    rng = np.random.default_rng(40 + window)
    V = 151936
    rule = B.TriggerRule(V, synth.modulo_bitmap(V, 97), synth.modulo_bitmap(V, 89), window)
    for n, lo, hi, cap in [(5000, 3, 4990, 4096), (300, 0, 300, 4096), (300, 100, 250, 2), (64, 0, 0, 0)]:
        toks = torch.from_numpy(_tokens(rng, n, V)).cuda()
        want_n, want_pos = B.st_trigger_scan(rule, toks, lo, hi, cap)
        got_n, got_pos = B.st_trigger_scan_static(rule, toks, lo, hi, cap)
        assert got_n == want_n and got_pos.tolist() == want_pos.tolist(), (n, lo, hi, cap)
        assert n < 1000 or want_n > 20                           # the large case really has hits to stage
    with pytest.raises(B.StError) as e:
        B.st_trigger_scan_static(rule, toks, 0, 64, B.ST_SCAN_STATIC_MAX_CAP + 1)
    assert e.value.code == B.ST_ERANGE
