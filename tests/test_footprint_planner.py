"""Footprint planner (host only): closed form, and a sanity range against the batch-size columns the paper prints
in Table 1.  The paper's batches are limited by weights and activations as well as by the KV cache, so only the
ORDER of the gain is compared: the KV-only gain L / slots must lie within the spread of the printed gains for the
1.1B and 7B models (for 30B the baseline fits 1-4 sequences next to the weights, so its printed gains are not a
KV-cache ratio)."""
import os

import numpy as np
import pytest

from paper_2405_10637_amd import binding as lk
from paper_2405_10637_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_batch_sizes.txt")
SHAPES = {"1.1B": dict(L=22, Hq=32, Hkv=4, D=64), "7B": dict(L=32, Hq=32, Hkv=32, D=128)}

pytestmark = pytest.mark.skipif(not os.path.exists(lk.LIB_PATH), reason="liblckv.so not built")


def cfg(model, w, T):
    s = SHAPES[model]
    return lk.make_config(s["L"], s["Hq"], s["Hkv"], s["D"], lk.LCKV_BF16, 1, T, synth.sandwich_mask(s["L"], w))


def test_planner_closed_form():
    T = 4096
    c = cfg("7B", 2, T)
    per_seq = 3 * T * 2 * 32 * 128 * 2                    # slots * T * 2 * Hkv * D * elem
    assert lk.lckv_cache_bytes(c) == per_seq
    for budget in (per_seq - 1, per_seq, 10 * per_seq + 5, 80 * 2 ** 30):
        assert lk.lckv_plan_max_batch(c, budget) == budget // per_seq
    # standard transformer: every layer keeps a cache
    assert lk.lckv_plan_max_batch(cfg("7B", 32, T), 80 * 2 ** 30) == (80 * 2 ** 30) // (32 * T * 2 * 32 * 128 * 2)


def test_kv_only_gain_lies_within_the_papers_printed_gains():
    printed = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            gpu, model, layers, seq, b0, b2, b10 = line.split()
            if model in SHAPES:
                printed.setdefault((model, 2), []).append(int(b2) / int(b0))
                printed.setdefault((model, 10), []).append(int(b10) / int(b0))
    budget = 64 * 2 ** 30
    for (model, w), gains in printed.items():
        T = 4096
        ours = lk.lckv_plan_max_batch(cfg(model, w, T), budget) / lk.lckv_plan_max_batch(
            cfg(model, SHAPES[model]["L"], T), budget)
        want = SHAPES[model]["L"] / (w + 1)
        assert abs(ours - want) / want < 0.02                 # L / slots, up to integer rounding of the batches
        assert min(gains) <= ours <= max(gains), (model, w, ours, gains)


def test_planner_rejects_paged_and_bad_configs():
    c = cfg("7B", 2, 4096)
    c.page_size, c.num_blocks = 16, 100
    with pytest.raises(lk.LckvError):
        lk.lckv_plan_max_batch(c, 1 << 30)
    c = cfg("7B", 2, 4096)
    c.D = 100
    with pytest.raises(lk.LckvError):
        lk.lckv_plan_max_batch(c, 1 << 30)
