"""The benchmark's CPU-baseline extrapolation counts work in (query head, key) visits; the count for a whole step
is checked here against a brute-force enumeration of every (layer, sequence, query head) item of a small workload
under the pairing of Section 2.1 (condensed layers see t_b keys, warmup layers t_b + 1)."""
import numpy as np

import bench
from oracle import lckv_oracle as orc
from paper_2405_10637_amd import synth


def brute_force_visits(wl, lens, step_index=0):
    _, vis, _ = orc.pairing(wl.warmup_mask)
    n = 0
    for l in range(wl.L):
        for b in range(wl.B):
            for _h in range(wl.Hq):
                n += int(lens[b]) + step_index + int(vis[l])
    return n


def test_key_visits_match_a_brute_force_count():
    for wl in (synth.C1, synth.C2.with_(B=3, T=40), synth.C4.with_(B=5, T=90, T_min=3, L=6, w=2),
               synth.C5.with_(B=2, T=17, L=8, w=4)):
        lens = synth.seq_lens(wl)
        _, vis, _ = orc.pairing(wl.warmup_mask)
        for step in (0, 3):
            assert bench.key_visits_per_step(lens, vis, wl.Hq, step) == brute_force_visits(wl, lens, step)


def test_visits_per_unit_is_the_units_own_key_count():
    # a sample of all units, each counted with its own keys, sums to the whole step: the ratio that scales the
    # sample's time is 1 when the sample is everything
    wl = synth.C2.with_(B=2, T=9, L=5, w=2)
    lens = synth.seq_lens(wl)
    _, vis, _ = orc.pairing(wl.warmup_mask)
    per_unit = [int(lens[b]) + int(vis[l]) for l in range(wl.L) for b in range(wl.B) for _ in range(wl.Hq)]
    assert sum(per_unit) == bench.key_visits_per_step(lens, vis, wl.Hq)
    assert len(per_unit) == wl.L * wl.B * wl.Hq
