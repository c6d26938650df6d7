"""The synthetic workloads carry the shapes the paper prints (appendix table "Model configurations") and
the sandwich placement of Section 2.1; lengths and block tables follow the stated recipe."""
import os

import numpy as np

from paper_2405_10637_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "model_shapes.txt")


def paper_shapes():
    rows = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            name, hidden, layers, heads, kv = line.split()
            rows[name] = dict(hidden=int(hidden), L=int(layers), Hq=int(heads), Hkv=int(kv))
    return rows


def test_workload_shapes_match_the_papers_table():
    shapes = paper_shapes()
    for wl, model in [(synth.C2, "1.1B"), (synth.C3, "7B"), (synth.C4, "7B")]:
        s = shapes[model]
        assert (wl.L, wl.Hq, wl.Hkv) == (s["L"], s["Hq"], s["Hkv"])
        assert wl.D == s["hidden"] // s["Hq"]


def test_sandwich_mask():
    assert synth.sandwich_mask(22, 2).nonzero()[0].tolist() == [0, 21]
    assert synth.sandwich_mask(40, 10).nonzero()[0].tolist() == [0, 1, 2, 3, 4, 35, 36, 37, 38, 39]
    assert synth.sandwich_mask(4, 0).sum() == 0 and synth.sandwich_mask(4, 4).sum() == 4
    assert synth.C1.warmup_mask.tolist() == [1, 0, 0, 0]


def test_ragged_lengths_and_block_table():
    lens = synth.seq_lens(synth.C4)
    assert lens.shape == (256,) and lens.min() >= 256 and lens.max() <= 8192
    assert (lens == synth.seq_lens(synth.C4)).all()                  # seeded
    assert 3500 < lens.mean() < 5000
    table, nb = synth.block_table(synth.C4, lens)
    need = (lens.astype(np.int64) + 1 + 15) // 16
    used = table[table >= 0]
    assert used.size == need.sum() == nb
    assert np.array_equal(np.sort(used), np.arange(nb))              # a permutation: no block shared
    for b in (0, 100, 255):
        assert (table[b, : need[b]] >= 0).all() and (table[b, need[b]:] == -1).all()
    assert not np.array_equal(used, np.arange(nb))                   # scattered, not in order


def test_inputs_are_seeded_and_in_dtype():
    q, k, v = synth.step_inputs(synth.C1, 2)
    q2, _, _ = synth.step_inputs(synth.C1, 2)
    assert q.dtype.is_floating_point and q.shape == (4, 2, 4, 64) and k.shape == (2, 2, 4, 64)
    assert (q == q2).all() and not (k == v).all()
    wl = synth.C2.with_(B=2, T=32)
    q, k, v = synth.step_inputs(wl, 3)
    assert str(q.dtype) == "torch.bfloat16" and 0.4 < q.float().std() < 0.6
